// Argument block and launchers of the persistent single-sample kernels (persistent_kernels.hip).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>

namespace lf {

constexpr int kMaxGroups = 256;          // chain workgroups of a persistent kernel (one per compute unit)
constexpr int kMaxRowsPerGroup = 256;    // rows one forward workgroup may own
constexpr int kMaxPersistentN = 4096;    // wider nets take the stream schedule
constexpr int kMaxPersistentDepth = 1025; // deeper nets too (the per-layer pointer tables live in LDS)
constexpr int kMaxRowSplit = 4;          // row blocks a backward column strip may be split into
constexpr int kMaxLaunchGroups = 1024;   // workgroups of one launch (chain + gradient workers)

struct PersistArgs {
    int L, N;                            // layers 2..L-1 have N neurons
    int n_in, n_out;                     // neurons of layer 1 and of layer L: multiples of 4, at most N
    int G, RPG;                          // forward: workgroups, rows per workgroup
    int GB, TPR;                         // backward chain: workgroups, float4 column groups per strip
    int RS;                              // backward chain: row blocks per strip (1 = a strip is one workgroup's)
    int GW, k;                           // gradient worker workgroups, worker partitions
    int workers;                         // 1 = the grid has gradient worker workgroups (k >= 2, or the descent
                                         // step is on); 0 = the chain workgroups form the gradients in line
    int fused;                           // 1 = on-chain fusion: the chain workgroups store nabla_w^{l+1} inside the
                                         // loop that multiplies w^{l+1} (a grid without workers)
    int no_grads;                        // 1 = the chain alone: no gradient is formed (a timing aid; a grid
                                         // without workers)
    int stream_weights;                  // 1 = the weights are too many to stay in the caches from one use to the
                                         // next: the wide-layer kernel instances read them with non-temporal loads
    int spread;                          // 1 = worker partitions span all XCDs when k is a multiple of 4 (see gradient_worker)
    int pace;                            // > 1: a worker stores a layer's rows in this many bursts, one per chain step
    int strip_run;                       // row-block strips: an XCD takes runs of this many adjacent strips (0: all of its strips adjacent)
    int fwd_band;                        // 1 = forward: an XCD owns a contiguous eighth of the rows (see forward_pass)
    float sgd_eta;                       // != 0: the workers apply w -= eta nabla_w, b -= eta nabla_b in place
    unsigned long long* reads_done;      // [L-1][kMaxGroups] tagged words, row l-2: chain workgroup g has
                                         // finished reading w^l (written only while the descent step is on)
    unsigned epoch;                      // tag of this launch's words (never 0): filled in by the kernel from its
                                         // workgroup's launch count (see launch_count)
    unsigned* counts_fwd;                // per-workgroup launch counts, kMaxLaunchGroups words each, all starting
    unsigned* counts_bwd1;               // at 1: forward grid, backward grid with k = 1, backward grid with
    unsigned* counts_bwdk;               // k >= 2
    float cost_scale;                    // power of two multiplied into delta^L (see lf_set_cost_scale)
    unsigned spin_limit;                 // polls after which a wait gives up and raises the abort word
    int nap;                             // pause before the first poll of an exchange, in units of 256 cycles
    int ll_shift;                        // exchanged vectors: element i is word ((i >> 3) << ll_shift) + (i & 7)
    size_t ll_layer;                     // and one layer's vector takes ll_layer words
    const float* const* w;               // device tables, index l-2
    const float* const* b;
    float* const* gw;
    float* const* gb;
    const float* a1;                     // x^1
    float* a_base;  size_t a_stride;     // a^l = a_base + (l-2)*a_stride  (floats), l >= 2
    float* d_base;  size_t d_stride;     // delta^l likewise
    unsigned long long* DLL;             // [L-1][ll_layer]  delta^l as tagged words
    unsigned long long* ALL;             // [L-1][ll_layer]  a^l as tagged words (forward)
    unsigned long long* PLL;             // [L-1][N][RS]  row-block partial sums of (bp2) as tagged words
    const float* y;
    int* abort_dev;                      // device word
    int* abort_host;                     // mapped pinned host word, or null
};

bool persistent_supported(int L, int N);
// Words one layer's exchanged vector of N elements takes when groups of eight words lie 8 << ll_shift
// bytes apart (ll_shift = 3: packed).
size_t persistent_ll_layer_words(int N, int ll_shift);
// Launch shapes for width N on a device with num_cus compute units; requested > 0 overrides the
// default number of workgroups.
void persistent_forward_shape(int N, int num_cus, int requested, int* G, int* rpg);
// row_split: 1, 2 or 4 row blocks per column strip, anything else = the default for this N.
void persistent_backward_shape(int N, int num_cus, int requested, int row_split, int* GB, int* tpr, int* rs);
// Workgroups of the forward / backward / fused backward kernel instance for A's shape that one compute unit
// holds at a time (the runtime's occupancy figure for that very instance).
hipError_t persistent_resident_per_cu(const PersistArgs& A, int* forward, int* backward, int* backward_fused);
hipError_t launch_fill_u64(void* p, size_t n_words, unsigned long long v, hipStream_t s);
hipError_t launch_fwd_persistent(const PersistArgs& A, hipStream_t s);
hipError_t launch_bwd_persistent(const PersistArgs& A, hipStream_t s);

}  // namespace lf
