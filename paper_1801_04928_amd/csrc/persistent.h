// Argument block and launchers of the persistent single-sample kernels (persistent_kernels.hip).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>

namespace lf {

constexpr int kMaxGroups = 256;          // workgroups of a persistent kernel (one per compute unit)
constexpr int kMaxRowsPerGroup = 256;    // rows/columns one workgroup may own
constexpr int kMaxPersistentN = 8192;

struct PersistArgs {
    int L, N, G, RPG, k;
    unsigned epoch;                      // tag of this launch's words (never 0)
    const float* const* w;               // device tables, index l-2
    const float* const* b;
    float* const* gw;
    float* const* gb;
    const float* a1;                     // x^1
    float* a_base;  size_t a_stride;     // a^l = a_base + (l-2)*a_stride  (floats), l >= 2
    float* d_base;  size_t d_stride;     // delta^l likewise
    unsigned long long* X;               // [2][G][N] partial column sums of the chain step
    unsigned long long* DLL;             // [L-1][N]  delta^l as tagged words
    unsigned long long* ALL;             // [L-1][N]  a^l as tagged words (forward)
    const float* y;
    int* abort_dev;                      // device word
    int* abort_host;                     // mapped pinned host word, or null
};

int persistent_groups(int N, int num_cus);
bool persistent_supported(int N);
int persistent_rows_per_group(int N, int G);
hipError_t launch_fill_u64(void* p, size_t n_words, unsigned long long v, hipStream_t s);
hipError_t launch_fwd_persistent(const PersistArgs& A, hipStream_t s);
hipError_t launch_bwd_persistent(const PersistArgs& A, hipStream_t s);

}  // namespace lf
