/* lf.h -- C ABI of the leapfrogging backpropagation library for one MI355X (gfx950).
 *
 * One full backpropagation pass through an L-layer, width-N, fully connected
 * sigmoid network, in the paper's notation (section 2): layers are numbered
 * 1..L, a^1 = x^1, weights w^l (N x N) and biases b^l (N) exist for l = 2..L.
 * The serial chain -- forward z^l = w^l a^{l-1} + b^l, a^l = sigma(z^l), and
 * backward delta^l = ((w^{l+1})^T delta^{l+1}) (.) sigma'(z^l) -- is computed
 * once; the gradient terms nabla_b^l = delta^l and nabla_w^l = delta^l (a^{l-1})^T
 * are taken off that chain and computed by k interleaved workers, worker
 * (L - l) mod k owning layer l (section 3, Algorithm 1).
 *
 * Conventions
 *   - Every `l` at this boundary is the paper's layer index, 2 <= l <= L.
 *     Arrays of per-layer pointers have L-1 entries; entry i belongs to layer i+2.
 *   - Matrices are row-major: w^l[j][k] = w[j*N + k] is the weight into neuron j
 *     of layer l from neuron k of layer l-1 (the index order of eq. (bp4)).
 *   - A minibatch of B samples is sample-major: x[b*N + n].  B = 1 is the paper's
 *     single-sample case.  With B > 1 the cost and both gradients are summed
 *     (not averaged) over the samples.
 *   - Storage type `dt` applies to w^l, x^1, y and the stored activations a^l.
 *     b^l, delta^l, nabla_b^l and nabla_w^l are always fp32.  All accumulation
 *     is fp32.  bfloat16 values are produced with round-to-nearest-even.
 *   - All data pointers are DEVICE pointers, 16-byte aligned, BORROWED: the
 *     caller owns every buffer (weights, inputs, workspace, gradient buffers)
 *     and keeps it alive while the handle uses it.  Arrays of pointers
 *     (`const void* const*`) are HOST arrays, read during the call only.
 *   - `hip_stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     lf_forward and lf_backward_leapfrog only enqueue work and return; the work
 *     is ordered on that stream: anything enqueued on it afterwards sees the
 *     finished results (the "join" of Algorithm 1).
 *     After the first pass of a handle with the same k (which sets the handle up, creates worker streams and
 *     may synchronise), lf_forward and lf_backward_leapfrog consist of kernel launches, event records and
 *     event waits only and may be recorded in a HIP graph, with either schedule (the worker streams fork
 *     from and join hip_stream through events); a replay gives the same results as the recorded calls would.
 *   - Every function returns an lf_status; nothing throws, nothing aborts.
 *     After a non-OK status lf_last_error() describes it.  A handle is not
 *     thread-safe.  Different handles share nothing, with one restriction: the persistent
 *     kernels (LF_SCHED_PERSISTENT, LF_SCHED_FUSED, and LF_SCHED_AUTO where it picks them: B = 1,
 *     fp32, layers 2..L-1 of one width N <= 4096, the first and last no wider) need every workgroup
 *     of a launch resident at once, because the
 *     workgroups wait for each other.  The library checks at set-up that the idle device holds them
 *     (the runtime's occupancy figure for the kernel); it cannot see what else runs.  So do not let
 *     such a pass overlap on the device with another kernel that holds compute units for long
 *     (another handle's persistent pass on a second stream, other libraries' kernels): enqueue them
 *     on one stream or order them with events.  If the workgroups starve anyway, every wait is
 *     bounded: the kernel drains, and the next call on the handle returns LF_EHIP with the place of
 *     the wait (after seconds, not a hang).  An LF_SCHED_AUTO handle then moves to the stream
 *     schedule for good and works again from the next lf_forward; a handle set to
 *     LF_SCHED_PERSISTENT or LF_SCHED_FUSED stays failed (destroy it).
 *   - Shape limits: N a multiple of 4 (fp32) or 8 (bf16) so rows stay 16-byte
 *     aligned; 2 <= L <= 4096; 1 <= B; 1 <= k <= L-1.
 *   - Layers of different widths (lf_create_widths): section 2 fixes N neurons per
 *     layer only for its cost analysis and notes that the equations hold in general.
 *     With n_l neurons in layer l, w^l and nabla_w^l are n_l x n_{l-1} (row-major,
 *     row stride n_{l-1}), b^l, nabla_b^l, a^l, delta^l have n_l entries per sample,
 *     x^1 is [B][n_1] and y is [B][n_L].  Every n_l obeys the limit on N above.
 */
#ifndef LF_H
#define LF_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    LF_OK = 0,
    LF_EINVAL = 1,        /* bad argument: shape, k, null or misaligned pointer, small workspace */
    LF_ESTATE = 2,        /* call out of order: parameters/buffers not set, backward before forward */
    LF_ENOMEM = 3,        /* host allocation failed */
    LF_EHIP = 4,          /* a HIP call failed (no device, launch error, ...) */
    LF_EUNSUPPORTED = 5   /* valid request the library cannot serve */
} lf_status;

/* (The last enumerator of each input enum only widens its range to that of int, so that a caller's
 * out-of-range value reaches the library's argument check as a value and not as undefined behaviour.) */
typedef enum { LF_F32 = 0, LF_BF16 = 1, LF_DTYPE_INT_RANGE = 0x7fffffff } lf_dtype;

/* Cost function C.  Section 2 names a cost function without fixing one; the library offers the
 * quadratic cost C = 1/2 sum_b ||a^L_b - y_b||^2, hence nabla_a^L C = a^L - y. */
typedef enum { LF_COST_QUADRATIC = 0, LF_COST_INT_RANGE = 0x7fffffff } lf_cost;

/* How the k workers of section 3 are realised on the one GPU. */
typedef enum {
    LF_SCHED_AUTO = 0,        /* the library picks (persistent where supported) */
    LF_SCHED_STREAMS = 1,     /* chain on the caller's stream, k worker streams fed by per-layer events */
    LF_SCHED_PERSISTENT = 2,  /* one persistent kernel, k workgroup partitions fed by per-layer ready flags */
    LF_SCHED_REDUNDANT = 3,   /* Algorithm 1 as printed, for comparison: the parent (the caller's stream) walks
                                 the top k layers, then each of k worker streams walks its OWN delta chain down
                                 from delta^{L-j}, recomputing every delta^l, and forms the gradients of every
                                 k-th layer.  Single sample, fp32, k <= 8; same results, bit for bit, as
                                 LF_SCHED_STREAMS (the same kernels); k times the chain's work */
    LF_SCHED_FUSED = 4,       /* no workers at all, for comparison with leapfrogging (eqs. (bp2), (bp4) and the
                                 cost analysis of section 4): the persistent chain kernel's thread that
                                 multiplies an entry of w^{l+1} into delta^l also stores the same entry of
                                 nabla_w^{l+1} = delta^{l+1} (a^l)^T in the same loop, so reads and writes
                                 alternate on the chain and f3 is paid there in full.  k is checked and
                                 otherwise ignored.  Same shapes as LF_SCHED_PERSISTENT; same results, bit for
                                 bit; not with lf_set_sgd */
    LF_SCHED_INT_RANGE = 0x7fffffff
} lf_sched;

/* Flags of lf_set_debug_flags. */
typedef enum {
    LF_DEBUG_CHAIN_ONLY = 1   /* lf_backward_leapfrog computes the delta chain (bp1), (bp2) alone: no worker runs,
                                 no nabla_b^l or nabla_w^l is formed, the gradient buffers keep what they held and
                                 lf_grads returns LF_ESTATE.  A timing aid: this is the term f2 of section 4,
                                 against which "the gradients are hidden behind the chain" is judged */
} lf_debug_flag;

typedef struct lf_net lf_net;   /* opaque handle */

/* Bytes of device workspace a net of this shape needs (activations a^2..a^L,
 * errors delta^2..delta^L, reduction partials, ready flags).  0 if the shape is
 * invalid. */
size_t lf_workspace_bytes(int L, int N, int B, lf_dtype dt);

/* Create a handle.  `workspace` is caller-owned device memory of at least
 * lf_workspace_bytes() bytes, 256-byte aligned; its contents need not be
 * initialised.  Pure host work: touches no device.  LF_EINVAL on a bad shape,
 * null/misaligned/small workspace. */
lf_status lf_create(lf_net** out, int L, int N, int B, lf_dtype dt, lf_cost cost,
                    void* workspace, size_t workspace_bytes);

/* The same two calls for a net whose layers differ in width (section 2: the equations are valid for any
 * widths).  n: HOST array of L entries, n[l-1] = neurons of layer l, read during the call only.  The
 * persistent kernels take a net whose layers 2..L-1 have one width and whose first and last layer are no
 * wider than that (an input and an output of their own sizes around equal hidden layers); any other net runs
 * the stream schedule (LF_SCHED_PERSISTENT is then LF_EUNSUPPORTED, LF_SCHED_AUTO picks streams).  With all
 * n[l-1] equal this is lf_create. */
size_t lf_workspace_bytes_widths(int L, const int* n, int B, lf_dtype dt);
lf_status lf_create_widths(lf_net** out, int L, const int* n, int B, lf_dtype dt, lf_cost cost,
                           void* workspace, size_t workspace_bytes);

/* Register w^l and b^l, l = 2..L (section 2).  w[i]: N*N elements of type dt;
 * b[i]: N floats (n_l x n_{l-1} and n_l for layer l = i+2 of a net made by lf_create_widths).  The pointers
 * are kept; the data may change between passes. */
lf_status lf_set_params(lf_net* net, const void* const* w, const void* const* b);

/* Register where nabla_w^l (N*N floats) and nabla_b^l (N floats) are written,
 * l = 2..L.  Each pass overwrites them (never accumulates). */
lf_status lf_set_grad_buffers(lf_net* net, float* const* nabla_w, float* const* nabla_b);

/* Select the worker realisation for later lf_backward_leapfrog calls.
 * LF_EUNSUPPORTED if the shape/type has no such path.  With LF_SCHED_REDUNDANT, lf_backward_leapfrog returns
 * LF_EUNSUPPORTED for k > 8 or while lf_set_sgd is on; with LF_SCHED_FUSED while lf_set_sgd is on. */
lf_status lf_set_schedule(lf_net* net, lf_sched sched);

/* Set the debug flags (an OR of lf_debug_flag values; 0, the default, clears them).  LF_EINVAL for unknown
 * bits.  With LF_DEBUG_CHAIN_ONLY a later lf_backward_leapfrog is LF_EUNSUPPORTED while lf_set_sgd is on or
 * the schedule is LF_SCHED_REDUNDANT. */
lf_status lf_set_debug_flags(lf_net* net, unsigned flags);

/* Multiply the cost by 2^log2_scale (default 0).  Eq. (bp1) then yields 2^log2_scale * delta^L and, since
 * eqs. (bp2)-(bp4) are linear in delta, every delta^l, nabla_b^l and nabla_w^l comes out multiplied by
 * the same power of two: exactly, as long as nothing overflows.  In deep sigmoid nets delta^l shrinks by
 * about 4x per layer and leaves the fp32 normal range after some 60 layers; a scale keeps the lower
 * layers' gradients at full precision (the caller divides by the scale, or folds it into the step size).
 * LF_EINVAL unless -126 <= log2_scale <= 127. */
lf_status lf_set_cost_scale(lf_net* net, int log2_scale);

/* Fuse a plain gradient-descent step into the workers.  The paper ends at the gradients of eqs. (bp3), (bp4);
 * this is the step that consumes them, taken by the worker that has just formed them so that nabla_w^l is
 * never written to memory and read back.  With eta > 0 every later lf_backward_leapfrog applies
 *     w^l <- w^l - eta nabla_w^l,   b^l <- b^l - eta nabla_b^l     (l = 2..L)
 * in place, in the buffers registered with lf_set_params (which must then be writable), and stores no
 * gradients: lf_set_grad_buffers is not needed and lf_grads returns LF_ESTATE.  Each gradient entry is
 * rounded to fp32 as it would have been stored, then applied with one fused multiply-add.  Layer l's step
 * waits until the chain has read w^l for delta^{l-1}.  After such a pass the stored a^l, delta^l still belong
 * to the old weights; the next backward pass needs a new lf_forward (else LF_ESTATE).
 * eta = 0 (default) switches it off.  Both schedules have it; they form delta^l with different (fixed)
 * summation orders, so the stepped weights of the two agree to rounding, not bit for bit.
 * bfloat16 storage: a step of eta nabla_w is mostly below half a unit of a bfloat16 weight, so the step is
 * taken on fp32 master copies (lf_set_master_weights; LF_ESTATE at the backward pass without them):
 * master <- master - eta nabla_w in fp32, and w^l is rewritten as the master rounded to nearest even.
 * LF_EINVAL unless eta is finite and >= 0. */
lf_status lf_set_sgd(lf_net* net, float eta);

/* Register fp32 master copies of the weights of a bfloat16 net (w32[i]: n_l x n_{l-1} floats for layer i+2,
 * device memory, caller-owned and caller-initialised, normally with the values w^l was rounded from).  Only
 * the fused descent step reads and writes them.  LF_EINVAL for an fp32 net, NULL or misaligned pointers. */
lf_status lf_set_master_weights(lf_net* net, float* const* w32);

/* Forward pass, eqs. (x), (z), (a): a^1 = x^1; for l = 2..L
 * z^l = w^l a^{l-1} + b^l, a^l = sigma(z^l).  x1: [B][N] of type dt, aliased as
 * a^1 (it must stay valid and unchanged until the backward pass has finished).
 * z^l is not stored (sigma' is formed from a^l). */
lf_status lf_forward(lf_net* net, const void* x1, void* hip_stream);

/* Backward pass with k interleaved workers (section 3, Algorithm 1).
 * Eq. (bp1) delta^L = (a^L - y) (.) sigma'(z^L); eq. (bp2) down the chain, once;
 * eqs. (bp3), (bp4) for layer l by worker (L - l) mod k as soon as delta^l is
 * ready.  k = 1 is the sequential pass (gradients in line with the chain).
 * The gradients do not depend on k, bit for bit.  y: [B][N] of type dt.
 * LF_ESTATE unless lf_forward has run since the last lf_set_params;
 * LF_EINVAL unless 1 <= k <= L-1. */
lf_status lf_backward_leapfrog(lf_net* net, const void* y, int k, void* hip_stream);

/* lf_backward_leapfrog for callers that cannot allocate: code that records the pass into a HIP graph on its
 * first call, tight serving loops, harnesses that forbid hipMalloc.  (lf_backward_leapfrog may create worker
 * streams and events, or pinned memory, the first time a handle runs with a new k or schedule.)  This call
 * allocates nothing, on the device or through any library: it enqueues the stream schedule's kernels -- chain
 * and gradient kernels of layer L, L-1, ..., 2 in that order -- on hip_stream alone, and the scratch of the chain
 * products (row-block partial sums at B = 1, split-K partials of a minibatch) is a static device array inside
 * the library instead of the caller's workspace.  Same arguments, same checks, same results bit for bit as
 * lf_backward_leapfrog with LF_SCHED_STREAMS (k only names the worker a layer would belong to; the gradients do
 * not depend on it).  lf_forward must have run (with LF_SCHED_STREAMS it allocates nothing either).
 * Limits: the chain scratch of the net's shape (a part of lf_workspace_bytes) must fit
 * lf_noalloc_scratch_limit() bytes -- 8 MiB: every B = 1 net up to N = 8192, small minibatch nets -- else
 * LF_EUNSUPPORTED, with both sizes in lf_last_error(); the handle's schedule
 * must be LF_SCHED_AUTO, LF_SCHED_STREAMS or LF_SCHED_PERSISTENT (which only matter to the other calls).
 * Every call on one GPU uses that GPU's one array: calls that overlap in time on one GPU (two streams, two
 * handles, two threads) race on it; order them on one stream or with events.  The array is held from the
 * first call on a GPU until the process ends. */
lf_status lf_backward_leapfrog_noalloc(lf_net* net, const void* y, int k, void* hip_stream);
size_t lf_noalloc_scratch_limit(void);

/* Device pointers to nabla_w^l and nabla_b^l of the last backward pass (the
 * registered buffers).  Valid to read once the stream of that pass has reached
 * the end of it.  LF_ESTATE if no backward pass has been enqueued. */
lf_status lf_grads(lf_net* net, int l, const float** nabla_w, const float** nabla_b);

/* Device pointers to the stored a^l ([B][N], type dt; l = 1..L, l = 1 is x^1) and
 * delta^l ([B][N] fp32; l = 2..L, NULL for l = 1).  For tests of the identity
 * nabla_w^l[j][k] = a^{l-1}_k delta^l_j (eq. (bp4)).  Either out pointer may be NULL. */
lf_status lf_activations(lf_net* net, int l, const void** a_l, const float** delta_l);

/* Worker that owns layer l's gradients with k workers: (L - l) mod k, the thread
 * rule of Algorithm 1 extended to the top k layers.  -1 on invalid arguments.
 * Pure host function. */
int lf_schedule_worker(int L, int k, int l);

/* Who saves layer l's gradients in Algorithm 1 as printed (LF_SCHED_REDUNDANT): the parent for the top k
 * layers L..L-k+1 (returned as k), thread (L - l) mod k below them.  -1 on invalid arguments.  Pure host
 * function. */
int lf_algorithm1_owner(int L, int k, int l);

/* Description of the last failure on this handle (or of the last failed
 * lf_create when net is NULL).  Owned by the library; never NULL. */
const char* lf_last_error(const lf_net* net);

/* Release the handle (streams, events; never the caller's buffers).  NULL is fine. */
void lf_destroy(lf_net* net);

#ifdef __cplusplus
}
#endif
#endif /* LF_H */
