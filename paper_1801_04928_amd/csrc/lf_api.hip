// C ABI of the library (see include/lf.h): handle, argument and state checks, workspace layout, and
// the stream realisation of the leapfrog schedule of section 3 / Algorithm 1:
//   - the delta chain (bp1),(bp2) runs once, on the caller's stream;
//   - after delta^l is enqueued an event is recorded; worker (L-l) mod k, a stream of its own, waits
//     for that event and computes (bp3),(bp4) of layer l;
//   - at the end the caller's stream waits for every worker (the join).
// With k = 1 the gradient kernels are enqueued in line on the caller's stream (sequential pass).
#include "../../include/lf.h"
#include "lf_internal.h"
#include "persistent.h"

#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <mutex>
#include <new>
#include <string>
#include <vector>

// Scratch of lf_backward_leapfrog_noalloc: device memory that exists from the moment the library is loaded, so
// that the call needs no allocation.  Every GPU the library runs on holds its own copy at its own address; in
// host code the name below is only a handle for hipGetSymbolAddress, never an address to hand to a kernel.
#define LF_STATIC_SCRATCH_BYTES (8u << 20)
static __device__ __align__(256) unsigned char scratch[LF_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
void* g_static_scratch[kMaxDevices];   // device address of `scratch` on each device; null = not asked yet
std::mutex g_static_scratch_mutex;

constexpr size_t kAlign = 256;
constexpr int kMaxL = 4096;
constexpr int kMaxWorkerStreams = 32;   // workers beyond this share streams (worker j -> stream j mod 32)
constexpr int kMaxRedundantWorkers = 8; // LF_SCHED_REDUNDANT: each worker has a delta chain (and scratch) of its own

size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

std::string g_create_error = "no error";

struct Layout {
    size_t a_off, a_stride;          // a^2..a^L
    size_t d_off, d_stride;          // delta^2..delta^L (fp32)
    size_t dbf_off, dbf_stride;      // bfloat16 copies of delta (bf16 nets only)
    size_t partial_off, partial_bytes;
    // LF_SCHED_REDUNDANT (single sample): per worker two delta vectors (one layer's and the next's) and a
    // partial buffer of its own
    size_t red_off, red_vec_bytes, red_stride;
    size_t raw_off, raw_bytes;
    // persistent single-sample path: tagged-word exchange buffers, pointer tables, abort word
    size_t dll_off, all_off, ll_words;   // [L-1][ll_layer] each
    size_t ll_layer; int ll_shift;       // words per layer; spacing of the eight-word groups
    size_t pll_off, pll_words;           // [L-1][N][kMaxRowSplit]
    size_t tab_off, tab_bytes;       // w, b, nabla_w, nabla_b pointer tables, L-1 entries each
    size_t abort_off;
    size_t counts_off;               // per-workgroup launch counts: 3 x kMaxLaunchGroups words
    size_t reads_off, reads_words;   // [L-1][kMaxGroups] tagged words: chain workgroup g has finished reading w^l
    size_t total;
};

// n[l-1] = neurons of layer l, l = 1..L
bool valid_shape(int L, const int* n, int B, lf_dtype dt) {
    if (L < 2 || L > kMaxL || !n || B < 1) return false;
    if (dt != LF_F32 && dt != LF_BF16) return false;
    for (int i = 0; i < L; ++i) {
        if (n[i] < 1 || n[i] % (dt == LF_BF16 ? 8 : 4) != 0) return false;
        if ((size_t)n[i] * (size_t)B > ((size_t)1 << 40)) return false;
    }
    return true;
}

int widest(int L, const int* n) {
    int m = n[0];
    for (int i = 1; i < L; ++i) m = std::max(m, n[i]);
    return m;
}

bool all_equal(int L, const int* n) {
    for (int i = 1; i < L; ++i)
        if (n[i] != n[0]) return false;
    return true;
}

// The shape the persistent kernels take: layers 2..L-1 all of the widest width, the first and the last layer
// no wider (any two widths when L = 2).
bool inner_layers_equal(int L, const int* n) {
    const int N = widest(L, n);
    for (int i = 1; i + 1 < L; ++i)
        if (n[i] != N) return false;
    return true;
}

bool single_sample_path(int N, int B, lf_dtype dt) { return B == 1 && dt == LF_F32 && N <= 16384; }

// Spacing of the eight-word groups of an exchanged vector: 8 << shift bytes.
// LF_PERSISTENT_LL_STRIDE (bytes, a power of two from 64 to 65536) overrides it for tuning; it is read
// whenever a layout is made, so it has to be the same for lf_workspace_bytes and lf_create.
int ll_spread_shift() {
    int bytes = 64;
    if (const char* e = std::getenv("LF_PERSISTENT_LL_STRIDE")) bytes = std::atoi(e);
    int shift = 3;
    while ((8 << shift) < bytes && shift < 13) ++shift;
    return shift;
}

// Every layer's a^l and delta^l get a slot sized for the widest layer (N).
Layout make_layout(int L, const int* n, int B, lf_dtype dt) {
    Layout y{};
    const int N = widest(L, n);
    const size_t M = (size_t)(L - 1), bn = (size_t)B * N;
    const size_t es = dt == LF_BF16 ? 2 : 4;
    size_t off = 0;
    y.a_off = off;   y.a_stride = align_up(bn * es);   off += M * y.a_stride;
    y.d_off = off;   y.d_stride = align_up(bn * 4);    off += M * y.d_stride;
    y.dbf_off = off; y.dbf_stride = dt == LF_BF16 ? align_up(bn * 2) : 0; off += M * y.dbf_stride;
    // scratch of the chain-side products, sized for the layer that needs most: the row-block partial sums
    // of the single-sample chain step, the split-K partials of the minibatch products
    size_t partial_floats = 0, raw_floats = 0;
    for (int l = 2; l <= L; ++l) {
        const int n_l = n[l - 1], n_prev = n[l - 2];
        if (single_sample_path(N, B, dt)) {
            if (l >= 3)   // the step delta^l -> delta^{l-1} reads w^l (n_l x n_prev)
                partial_floats = std::max(partial_floats, (size_t)lf::chain_partial_blocks(n_l) * n_prev);
        } else {
            raw_floats = std::max(raw_floats, lf::split_workspace_floats(n_l, n_prev, B, dt == LF_BF16));
            if (l >= 3) raw_floats = std::max(raw_floats, lf::split_workspace_floats(n_prev, n_l, B, dt == LF_BF16));
        }
    }
    y.partial_off = off;
    y.partial_bytes = align_up(partial_floats * 4);
    off += y.partial_bytes;
    y.raw_off = off;
    y.raw_bytes = align_up(raw_floats * 4);
    off += y.raw_bytes;
    if (single_sample_path(N, B, dt)) {
        y.red_vec_bytes = align_up((size_t)N * 4);
        y.red_stride = 2 * y.red_vec_bytes + y.partial_bytes;
        y.red_off = off;
        off += kMaxRedundantWorkers * y.red_stride;
    }
    if (inner_layers_equal(L, n) && single_sample_path(N, B, dt) && lf::persistent_supported(L, N)) {
        y.ll_shift = ll_spread_shift();
        y.ll_layer = lf::persistent_ll_layer_words(N, y.ll_shift);
        y.ll_words = M * y.ll_layer;
        y.dll_off = off; off += align_up(y.ll_words * 8);
        y.all_off = off; off += align_up(y.ll_words * 8);
        y.pll_words = M * (size_t)N * lf::kMaxRowSplit;
        y.pll_off = off; off += align_up(y.pll_words * 8);
        y.tab_off = off; y.tab_bytes = 4 * M * sizeof(void*);         off += align_up(y.tab_bytes);
        y.abort_off = off; off += kAlign;
        y.counts_off = off; off += align_up(3 * lf::kMaxLaunchGroups * sizeof(unsigned));
        y.reads_words = M * lf::kMaxGroups;
        y.reads_off = off; off += align_up(y.reads_words * 8);
    }
    y.total = off;
    return y;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

struct lf_net {
    int L, N, B;                       // N: the widest layer
    std::vector<int> n;                // n[l-1] = neurons of layer l
    bool uniform;                      // every layer has N neurons
    bool inner_uniform;                // layers 2..L-1 have N neurons (the first and the last may have fewer)
    int width(int l) const { return n[l - 1]; }
    lf_dtype dt;
    lf_cost cost;
    lf_sched sched;
    float cost_scale;
    float sgd_eta;                     // != 0: the workers apply the descent step instead of storing gradients
    lf::GemmPlan gemm;                 // minibatch: which matrix kernels the products take (decided at creation)
    char* ws;
    Layout lay;
    std::vector<const void*> w;       // index l-2
    std::vector<const float*> b;
    std::vector<float*> gw, gb;
    std::vector<float*> w32;           // bfloat16 nets: fp32 master copies of w^l for the fused descent step
    bool have_master;
    const void* x1;
    bool have_params, have_grads, fwd_done, bwd_done;
    bool stepped;                      // a fused descent step has changed the weights since the last forward pass
    std::vector<hipStream_t> workers;
    std::vector<hipEvent_t> ev_delta;  // index l-2
    std::vector<hipEvent_t> ev_done;   // per worker stream
    std::string err;
    // persistent path
    unsigned debug_flags;              // LF_DEBUG_*
    bool p_ready, p_tables_dirty;
    bool p_failed_over;                // LF_SCHED_AUTO: a persistent wait gave up; the handle has moved to streams
    bool p_fused_ok;                   // the fused backward kernel's workgroups all fit the device at once
    int p_groups, p_rpg, p_bgroups, p_tpr, p_rs, p_workers, p_spread, p_pace, p_strip_run, p_fwd_band, p_nap_fwd, p_nap_bwd;
    unsigned p_spin_limit;             // polls before a bounded wait gives up
    int* p_abort_host;                 // pinned, mapped; the kernels raise it when a wait gives up
    int* p_abort_dev_view;             // the same word as the device addresses it
    std::vector<const void*> p_tables;

    void* a_ptr(int l) const {         // l = 1..L
        return l == 1 ? const_cast<void*>(x1) : ws + lay.a_off + (size_t)(l - 2) * lay.a_stride;
    }
    float* d_ptr(int l) const { return reinterpret_cast<float*>(ws + lay.d_off + (size_t)(l - 2) * lay.d_stride); }
    void* dbf_ptr(int l) const {
        return dt == LF_BF16 ? ws + lay.dbf_off + (size_t)(l - 2) * lay.dbf_stride : nullptr;
    }
    float* partial() const { return reinterpret_cast<float*>(ws + lay.partial_off); }
    float* raw() const { return lay.raw_bytes ? reinterpret_cast<float*>(ws + lay.raw_off) : nullptr; }
};

namespace {

// Whether a single-sample fp32 net's weights are far too many to stay in the device's 256 MB cache from the forward
// to the backward pass and from one pass to the next (then they are read with non-temporal loads).  Measured: 4.2 GB
// of weights gain 7 % forward and 2 % backward, 268 MB lose 10 % (part of them still hits), 130 MB lose a third; the
// line is drawn at twice the cache.  LF_PERSISTENT_STREAM_WEIGHTS=0/1 overrides.
bool weights_exceed_cache(const lf_net* net) {
    if (const char* e = std::getenv("LF_PERSISTENT_STREAM_WEIGHTS")) return e[0] == '1';
    size_t bytes = 0;
    for (int l = 2; l <= net->L; ++l) bytes += (size_t)net->width(l) * (size_t)net->width(l - 1) * sizeof(float);
    return bytes > (size_t)512 << 20;
}


lf_status fail(lf_net* net, lf_status st, const std::string& msg) {
    if (net) net->err = msg; else g_create_error = msg;
    return st;
}

lf_status fail_hip(lf_net* net, hipError_t e, const char* what) {
    return fail(net, LF_EHIP, std::string(what) + ": " + hipGetErrorString(e));
}

#define LF_HIP(net, call)                                         \
    do {                                                          \
        hipError_t e_ = (call);                                   \
        if (e_ != hipSuccess) return fail_hip(net, e_, #call);    \
    } while (0)

// Per-layer events, and `want` worker streams with an end-of-work event each.
lf_status ensure_worker_streams(lf_net* net, size_t want) {
    const size_t M = (size_t)net->L - 1;
    while (net->ev_delta.size() < M) {
        hipEvent_t e;
        LF_HIP(net, hipEventCreateWithFlags(&e, hipEventDisableTiming));
        net->ev_delta.push_back(e);
    }
    while (net->workers.size() < want) {
        hipStream_t s;
        LF_HIP(net, hipStreamCreateWithFlags(&s, hipStreamNonBlocking));
        net->workers.push_back(s);
        hipEvent_t e;
        LF_HIP(net, hipEventCreateWithFlags(&e, hipEventDisableTiming));
        net->ev_done.push_back(e);
    }
    return LF_OK;
}

// The stream schedule's workers: k streams (none for the sequential pass, which runs on the caller's).
lf_status ensure_workers(lf_net* net, int k) {
    // Workers beyond the plan's number of streams share them: worker j runs on stream j mod that number.
    // LF_WORKER_STREAMS overrides it (tuning).
    int cap = single_sample_path(net->N, net->B, net->dt) ? kMaxWorkerStreams
                                                          : std::min(kMaxWorkerStreams, net->gemm.worker_streams);
    if (const char* e = std::getenv("LF_WORKER_STREAMS")) {
        const int v = std::atoi(e);
        if (v >= 1 && v <= kMaxWorkerStreams) cap = v;
    }
    return ensure_worker_streams(net, k > 1 ? (size_t)(k < cap ? k : cap) : 0);
}

bool persistent_possible(const lf_net* net) {
    return net->inner_uniform && single_sample_path(net->N, net->B, net->dt) &&
           lf::persistent_supported(net->L, net->N);
}

bool use_persistent(const lf_net* net) {
    if (net->sched == LF_SCHED_FUSED) return true;           // (lf_set_schedule has checked the shape)
    if (net->sched == LF_SCHED_STREAMS || net->sched == LF_SCHED_REDUNDANT) return false;
    if (net->sched == LF_SCHED_AUTO && net->p_failed_over) return false;
    return persistent_possible(net);
}


// A persistent kernel whose wait gave up has raised the pinned abort word.
lf_status check_abort(lf_net* net) {
    const int code = net->p_abort_host ? *reinterpret_cast<volatile int*>(net->p_abort_host) : 0;
    if (code) {
        static const char* const site[] = {"partial-sum wait", "forward gather", "chain gather", "gradient wait"};
        std::string msg = std::string("a persistent kernel gave up waiting for its peers (") + site[(code >> 24) & 3] +
                          ", layer " + std::to_string((code >> 10) & 0x3fff) + ", workgroup " +
                          std::to_string(code & 0x3ff) + "); results are invalid";
        if (net->sched == LF_SCHED_AUTO) {
            // The library chose the persistent kernels; something else holds the compute units they need.
            // This call reports the lost pass, later passes of the handle take the stream schedule.
            *reinterpret_cast<volatile int*>(net->p_abort_host) = 0;
            net->p_failed_over = true;
            net->fwd_done = net->bwd_done = false;
            msg += "; the handle takes the stream schedule from now on (run lf_forward again)";
        }
        return fail(net, LF_EHIP, msg);
    }
    return LF_OK;
}

// One-time device set-up of the persistent path, and upload of the pointer tables when they changed.
lf_status prepare_persistent(lf_net* net, hipStream_t s) {
    if (!net->p_ready) {
        int dev = 0, cus = 0;
        LF_HIP(net, hipGetDevice(&dev));
        LF_HIP(net, hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
        // LF_PERSISTENT_GROUPS / LF_PERSISTENT_GROUPS_BWD: tuning overrides of the chain workgroup counts
        const char* env = std::getenv("LF_PERSISTENT_GROUPS");
        const char* envb = std::getenv("LF_PERSISTENT_GROUPS_BWD");
        lf::persistent_forward_shape(net->N, cus, env ? std::atoi(env) : 0, &net->p_groups, &net->p_rpg);
        // LF_PERSISTENT_ROW_SPLIT: row blocks per backward column strip (1, 2 or 4)
        const char* envr = std::getenv("LF_PERSISTENT_ROW_SPLIT");
        lf::persistent_backward_shape(net->N, cus, envb ? std::atoi(envb) : (env ? std::atoi(env) : 0),
                                      envr ? std::atoi(envr) : 0, &net->p_bgroups, &net->p_tpr, &net->p_rs);
        // LF_PERSISTENT_SPIN_LIMIT: polls before a bounded wait gives up (default 4M, i.e. seconds).  A
        // tiny value makes the first unlucky poll fail: the way to exercise the failure path in a test.
        const char* envs = std::getenv("LF_PERSISTENT_SPIN_LIMIT");
        net->p_spin_limit = envs ? (unsigned)std::strtoul(envs, nullptr, 10) : (4u << 20);
        net->p_workers = cus < lf::kMaxGroups ? cus : lf::kMaxGroups;
        // LF_PERSISTENT_WORKERS: tuning override of the number of gradient worker workgroups
        if (const char* envw = std::getenv("LF_PERSISTENT_WORKERS")) {
            const int w = std::atoi(envw);
            if (w >= 1 && w <= 2 * lf::kMaxGroups) net->p_workers = w;
        }
        if (net->p_workers > net->N) net->p_workers = net->N;
        // LF_PERSISTENT_SPREAD=0: worker partitions by workgroup index mod k for every k (a tuning knob; the
        // default gives every partition members on all XCDs when k is a multiple of 4)
        const char* envsp = std::getenv("LF_PERSISTENT_SPREAD");
        net->p_spread = (envsp && envsp[0] == '0') ? 0 : 1;
        // LF_PERSISTENT_PACE: bursts in which a worker stores a layer's rows, one per chain step (0 = all at once;
        // at most k; default k for nets whose weights exceed the cache, else 0)
        const char* envfb = std::getenv("LF_PERSISTENT_FWD_BAND");
        net->p_fwd_band = envfb ? (envfb[0] == '1' ? 1 : 0) : -1;
        const char* envm = std::getenv("LF_PERSISTENT_STRIP_RUN");
        net->p_strip_run = envm ? std::atoi(envm) : 0;
        if (net->p_strip_run < 0 || net->p_strip_run > 64) net->p_strip_run = 0;
        const char* envp = std::getenv("LF_PERSISTENT_PACE");
        net->p_pace = envp ? std::atoi(envp) : -1;
        if (net->p_pace < -1) net->p_pace = -1;
        // LF_PERSISTENT_NAP_FWD / _BWD: pause before the first poll of an exchange, units of 256 cycles
        const char* envnf = std::getenv("LF_PERSISTENT_NAP_FWD");
        const char* envnb = std::getenv("LF_PERSISTENT_NAP_BWD");
        // (measured best: about N/256 units forward, twice that backward, where a step does more work)
        int nap = net->N / 256;
        nap = nap < 2 ? 2 : (nap > 8 ? 8 : nap);
        net->p_nap_fwd = envnf ? std::atoi(envnf) : nap;
        net->p_nap_bwd = envnb ? std::atoi(envnb) : 2 * nap;
        if (net->p_nap_fwd < 0 || net->p_nap_fwd > 1024) net->p_nap_fwd = 0;
        if (net->p_nap_bwd < 0 || net->p_nap_bwd > 1024) net->p_nap_bwd = 0;
        // Every workgroup of a launch waits for others of it, so all of them must be resident at once: the
        // runtime's occupancy figure for the very kernel instances this shape takes says how many fit.
        if (net->p_rpg > lf::kMaxRowsPerGroup)
            return fail(net, LF_EUNSUPPORTED, "persistent path: too few compute units for this N");
        {
            lf::PersistArgs probe{};
            probe.L = net->L; probe.N = net->N;
            probe.n_in = net->width(1); probe.n_out = net->width(net->L);
            probe.G = net->p_groups; probe.RPG = net->p_rpg;
            probe.GB = net->p_bgroups; probe.TPR = net->p_tpr; probe.RS = net->p_rs;
            probe.stream_weights = weights_exceed_cache(net) ? 1 : 0;
            int occ_f = 0, occ_b = 0, occ_bf = 0;
            LF_HIP(net, lf::persistent_resident_per_cu(probe, &occ_f, &occ_b, &occ_bf));
            if (cus <= 0 || net->p_groups > occ_f * cus || net->p_bgroups + 1 > occ_b * cus)
                return fail(net, LF_EUNSUPPORTED, "persistent path: the device cannot hold all workgroups of a launch at once");
            if (net->p_workers > occ_b * cus - net->p_bgroups) net->p_workers = occ_b * cus - net->p_bgroups;
            net->p_fused_ok = net->p_bgroups <= occ_bf * cus;
        }
        if (!net->p_abort_host) {
            void* h = nullptr;
            LF_HIP(net, hipHostMalloc(&h, sizeof(int), hipHostMallocMapped));
            net->p_abort_host = static_cast<int*>(h);
            *net->p_abort_host = 0;
            void* d = nullptr;
            LF_HIP(net, hipHostGetDevicePointer(&d, h, 0));
            net->p_abort_dev_view = static_cast<int*>(d);
        }
        // tagged words start as tag 0 (never a valid tag); the abort word as 0
        LF_HIP(net, lf::launch_fill_u64(net->ws + net->lay.dll_off, net->lay.ll_words, 0ull, s));
        LF_HIP(net, lf::launch_fill_u64(net->ws + net->lay.all_off, net->lay.ll_words, 0ull, s));
        LF_HIP(net, lf::launch_fill_u64(net->ws + net->lay.pll_off, net->lay.pll_words, 0ull, s));
        LF_HIP(net, lf::launch_fill_u64(net->ws + net->lay.abort_off, kAlign / 8, 0ull, s));
        LF_HIP(net, lf::launch_fill_u64(net->ws + net->lay.reads_off, net->lay.reads_words, 0ull, s));
        // every workgroup's launch count starts at 1
        LF_HIP(net, lf::launch_fill_u64(net->ws + net->lay.counts_off, 3 * lf::kMaxLaunchGroups / 2,
                                        0x0000000100000001ull, s));
        net->p_ready = true;
    }
    if (net->p_tables_dirty) {
        const size_t M = (size_t)net->L - 1;
        net->p_tables.resize(4 * M);
        for (size_t i = 0; i < M; ++i) {
            net->p_tables[i] = net->w[i];
            net->p_tables[M + i] = net->b[i];
            net->p_tables[2 * M + i] = net->gw[i];
            net->p_tables[3 * M + i] = net->gb[i];
        }
        // ordered on the stream behind any kernel that still reads the old tables
        LF_HIP(net, hipMemcpyAsync(net->ws + net->lay.tab_off, net->p_tables.data(), net->lay.tab_bytes,
                                   hipMemcpyHostToDevice, s));
        LF_HIP(net, hipStreamSynchronize(s));   // the staging vector may be rewritten after return
        net->p_tables_dirty = false;
    }
    return LF_OK;
}

lf::PersistArgs persist_args(lf_net* net, const void* y, int k) {
    const size_t M = (size_t)net->L - 1;
    lf::PersistArgs A{};
    A.L = net->L; A.N = net->N;
    A.n_in = net->width(1); A.n_out = net->width(net->L);
    A.G = net->p_groups; A.RPG = net->p_rpg;
    A.GB = net->p_bgroups; A.TPR = net->p_tpr; A.RS = net->p_rs;
    A.GW = net->p_workers;
    A.k = k < net->p_workers ? k : net->p_workers;   // never more partitions than worker workgroups
    A.sgd_eta = net->sgd_eta;
    A.stream_weights = weights_exceed_cache(net) ? 1 : 0;
    A.spread = net->p_spread;
    A.fused = net->sched == LF_SCHED_FUSED ? 1 : 0;
    A.no_grads = (net->debug_flags & LF_DEBUG_CHAIN_ONLY) ? 1 : 0;
    A.workers = ((A.k > 1 || A.sgd_eta != 0.0f) && !A.fused && !A.no_grads) ? 1 : 0;
    // bursts per layer of a worker's stores: one per chain step for nets bound by memory (see gradient_worker)
    A.pace = net->p_pace >= 0 ? net->p_pace : (A.stream_weights ? A.k : 0);
    if (A.pace > A.k) A.pace = A.k;                          // a partition's next layer comes k steps later
    if (!A.workers || A.sgd_eta != 0.0f) A.pace = 0;
    // (LF_PERSISTENT_FWD_BAND=0/1 and LF_PERSISTENT_STRIP_RUN=1/2/4/8 override, tuning knobs)
    A.fwd_band = net->p_fwd_band >= 0 ? net->p_fwd_band : A.stream_weights;
    A.strip_run = net->p_strip_run > 0 ? net->p_strip_run : 2;
    A.reads_done = reinterpret_cast<unsigned long long*>(net->ws + net->lay.reads_off);
    A.epoch = 0;                                            // set by the kernel
    A.counts_fwd = reinterpret_cast<unsigned*>(net->ws + net->lay.counts_off);
    A.counts_bwd1 = A.counts_fwd + lf::kMaxLaunchGroups;
    A.counts_bwdk = A.counts_bwd1 + lf::kMaxLaunchGroups;
    A.cost_scale = net->cost_scale;
    A.spin_limit = net->p_spin_limit;
    void** tab = reinterpret_cast<void**>(net->ws + net->lay.tab_off);
    A.w = reinterpret_cast<const float* const*>(tab);
    A.b = reinterpret_cast<const float* const*>(tab + M);
    A.gw = reinterpret_cast<float* const*>(tab + 2 * M);
    A.gb = reinterpret_cast<float* const*>(tab + 3 * M);
    A.a1 = static_cast<const float*>(net->x1);
    A.a_base = reinterpret_cast<float*>(net->ws + net->lay.a_off);  A.a_stride = net->lay.a_stride / 4;
    A.d_base = reinterpret_cast<float*>(net->ws + net->lay.d_off);  A.d_stride = net->lay.d_stride / 4;
    A.DLL = reinterpret_cast<unsigned long long*>(net->ws + net->lay.dll_off);
    A.ALL = reinterpret_cast<unsigned long long*>(net->ws + net->lay.all_off);
    A.PLL = reinterpret_cast<unsigned long long*>(net->ws + net->lay.pll_off);
    A.ll_shift = net->lay.ll_shift; A.ll_layer = net->lay.ll_layer;
    A.y = static_cast<const float*>(y);
    A.abort_dev = reinterpret_cast<int*>(net->ws + net->lay.abort_off);
    A.abort_host = net->p_abort_dev_view;
    return A;
}

// (bp3),(bp4) of layer l on stream s; with the descent step fused in, applied to w^l and b^l in place.
lf_status enqueue_grads(lf_net* net, int l, hipStream_t s, bool whole_chip = true) {
    const int i = l - 2;
    const bool sgd = net->sgd_eta != 0.0f, bf = net->dt == LF_BF16;
    float* out_w = !sgd ? net->gw[i] : (bf ? net->w32[i] : static_cast<float*>(const_cast<void*>(net->w[i])));
    float* out_b = sgd ? const_cast<float*>(net->b[i]) : net->gb[i];
    void* w_bf = (sgd && bf) ? const_cast<void*>(net->w[i]) : nullptr;
    if (single_sample_path(net->N, net->B, net->dt)) {
        LF_HIP(net, lf::launch_grad_outer_f32(net->d_ptr(l), static_cast<const float*>(net->a_ptr(l - 1)),
                                              out_w, out_b, net->width(l), net->width(l - 1), net->sgd_eta, s));
    } else {
        LF_HIP(net, lf::launch_grad_gemm(net->d_ptr(l), net->dbf_ptr(l), net->a_ptr(l - 1), out_w, out_b,
                                         net->width(l), net->width(l - 1), net->B, bf, net->gemm, whole_chip,
                                         net->sgd_eta, w_bf, s));
    }
    return LF_OK;
}

// The same on worker (L - l) mod k, once `ready` (an event recorded on the chain's stream) has passed.
lf_status enqueue_grads_on_worker(lf_net* net, int l, int k, int nstreams, hipEvent_t ready, bool* used) {
    const int j = lf_schedule_worker(net->L, k, l) % nstreams;
    LF_HIP(net, hipStreamWaitEvent(net->workers[j], ready, 0));
    used[j] = true;
    // The last two gradient products (layers 3 and 2) run when the chain has all but ended: they take the whole
    // chip instead of the workers' share (configuration 5: 7.26 -> 7.18 ms on one box, two runs each).
    return enqueue_grads(net, l, net->workers[j], /*whole_chip=*/l <= 3);
}

// Algorithm 1 as printed (single sample).  The parent -- the caller's stream -- applies (bp1) and then
// (bp2),(bp3),(bp4) down to layer L-k+1; thread j, a stream of its own, starts from delta^{L-j}, walks the rest of
// the chain by itself and applies (bp3),(bp4) at layers L-k-j, L-2k-j, ...  A thread's delta^l goes to the
// net's delta^l slot when the thread owns layer l (nobody else writes that slot) and to one of the thread's two
// private vectors otherwise, so no two streams ever write the same memory.
lf_status backward_redundant(lf_net* net, const void* y, int k, hipStream_t s) {
    const int L = net->L;
    if (k > kMaxRedundantWorkers)
        return fail(net, LF_EUNSUPPORTED, "lf_backward_leapfrog: LF_SCHED_REDUNDANT has chains for at most 8 workers");
    if (net->sgd_eta != 0.0f)
        return fail(net, LF_EUNSUPPORTED, "lf_backward_leapfrog: LF_SCHED_REDUNDANT does not take the descent step");
    lf_status st = ensure_worker_streams(net, (size_t)k);       // a stream per thread, also for k = 1
    if (st != LF_OK) return st;
    auto chain = [&](int l, const float* d_next, float* d_l, float* partial, hipStream_t q) -> hipError_t {
        return lf::launch_chain_gemvT_f32(static_cast<const float*>(net->w[l - 1]), d_next,
                                          static_cast<const float*>(net->a_ptr(l)), d_l, partial,
                                          net->width(l + 1), net->width(l), q);
    };
    // parent
    LF_HIP(net, lf::launch_output_error(net->a_ptr(L), y, net->d_ptr(L), nullptr, (size_t)net->width(L), false,
                                        net->cost_scale, s));
    st = enqueue_grads(net, L, s);
    if (st != LF_OK) return st;
    const int parent_low = L - k + 1 > 2 ? L - k + 1 : 2;        // the parent's lowest layer
    for (int l = L - 1; l >= parent_low; --l) {
        LF_HIP(net, chain(l, net->d_ptr(l + 1), net->d_ptr(l), net->partial(), s));
        st = enqueue_grads(net, l, s);
        if (st != LF_OK) return st;
    }
    if (parent_low == 2) return LF_OK;                           // k = L-1: nothing is left for the threads
    // fork: the threads' seeds delta^L .. delta^{L-k+1} are all there once the parent is
    LF_HIP(net, hipEventRecord(net->ev_delta[0], s));
    for (int j = 0; j < k; ++j) {
        // thread j's layers are those below the parent's with (L - l) mod k = j; it walks down to the lowest
        // of them and no further (whole blocks of k layers, as in the algorithm's inner loop)
        const int lowest = 2 + ((L - j - 2) % k + k) % k;
        if (lowest > L - k) continue;                             // no layer of its own: the thread does nothing
        hipStream_t q = net->workers[j];
        LF_HIP(net, hipStreamWaitEvent(q, net->ev_delta[0], 0));
        char* mine = net->ws + net->lay.red_off + (size_t)j * net->lay.red_stride;
        float* vec[2] = {reinterpret_cast<float*>(mine), reinterpret_cast<float*>(mine + net->lay.red_vec_bytes)};
        float* partial = reinterpret_cast<float*>(mine + 2 * net->lay.red_vec_bytes);
        const float* cur = net->d_ptr(L - j);
        for (int l = L - j - 1; l >= lowest; --l) {
            const bool owned = lf_algorithm1_owner(L, k, l) == j;
            float* out = owned ? net->d_ptr(l) : vec[l & 1];
            LF_HIP(net, chain(l, cur, out, partial, q));
            if (owned) {
                st = enqueue_grads(net, l, q);
                if (st != LF_OK) return st;
            }
            cur = out;
        }
        LF_HIP(net, hipEventRecord(net->ev_done[j], q));
        LF_HIP(net, hipStreamWaitEvent(s, net->ev_done[j], 0));   // the join
    }
    return LF_OK;
}

// Argument and state checks shared by the backward entry points.
lf_status check_backward_call(lf_net* net, const void* y, int k) {
    if (!y) return fail(net, LF_EINVAL, "lf_backward_leapfrog: y is NULL");
    if (!aligned16(y)) return fail(net, LF_EINVAL, "lf_backward_leapfrog: y must be 16-byte aligned");
    if (k < 1 || k > net->L - 1) return fail(net, LF_EINVAL, "lf_backward_leapfrog: need 1 <= k <= L-1");
    if (!net->have_params) return fail(net, LF_ESTATE, "lf_backward_leapfrog: call lf_set_params first");
    if (!net->have_grads && net->sgd_eta == 0.0f)
        return fail(net, LF_ESTATE, "lf_backward_leapfrog: call lf_set_grad_buffers first");
    if (net->sgd_eta != 0.0f && net->dt == LF_BF16 && !net->have_master)
        return fail(net, LF_ESTATE, "lf_backward_leapfrog: lf_set_sgd on a bf16 net needs lf_set_master_weights");
    if (!net->fwd_done) return fail(net, LF_ESTATE, "lf_backward_leapfrog: call lf_forward first");
    if (net->stepped)
        return fail(net, LF_ESTATE, "lf_backward_leapfrog: the weights have been stepped since lf_forward; run it again");
    if ((net->debug_flags & LF_DEBUG_CHAIN_ONLY) && net->sgd_eta != 0.0f)
        return fail(net, LF_EUNSUPPORTED, "lf_backward_leapfrog: LF_DEBUG_CHAIN_ONLY and lf_set_sgd exclude each other");
    return LF_OK;
}

// The stream realisation of the schedule.  The chain runs on s; `partial` / `raw` are the scratch of its
// products (the row-block partial sums of the single-sample step, the split-K partials of the minibatch
// products).  in_line: layer l's gradient kernels follow delta^l on s itself (the sequential pass; also the
// entry point that may not create streams); otherwise worker (L - l) mod k's stream takes them behind an event.
lf_status backward_streams(lf_net* net, const void* y, int k, hipStream_t s, float* partial, float* raw,
                           bool in_line) {
    const int L = net->L, N = net->N, B = net->B;
    const bool bf = net->dt == LF_BF16;
    const bool b1 = single_sample_path(N, B, net->dt);
    const bool chain_only = (net->debug_flags & LF_DEBUG_CHAIN_ONLY) != 0;
    const bool sgd = net->sgd_eta != 0.0f;
    const int nstreams = in_line ? 0 : ((int)net->workers.size() < k ? (int)net->workers.size() : k);
    bool used[kMaxWorkerStreams] = {};
    lf_status st = LF_OK;
    for (int l = L; l >= 2; --l) {
        // the chain: (bp1) at L, (bp2) below
        if (l == L) {
            LF_HIP(net, lf::launch_output_error(net->a_ptr(L), y, net->d_ptr(L), net->dbf_ptr(L),
                                                (size_t)B * net->width(L), bf, net->cost_scale, s));
        } else if (b1) {
            // w^{l+1} has n_{l+1} rows and n_l columns
            LF_HIP(net, lf::launch_chain_gemvT_f32(static_cast<const float*>(net->w[l - 1]), net->d_ptr(l + 1),
                                                   static_cast<const float*>(net->a_ptr(l)), net->d_ptr(l),
                                                   partial, net->width(l + 1), net->width(l), s));
        } else {
            LF_HIP(net, lf::launch_chain_gemm(net->w[l - 1], net->d_ptr(l + 1), net->dbf_ptr(l + 1), net->a_ptr(l),
                                              net->d_ptr(l), net->dbf_ptr(l), raw, net->width(l),
                                              net->width(l + 1), B, bf, net->gemm, s));
        }
        // (bp3),(bp4) of layer l, off the chain: as soon as delta^l is there.  With the descent step fused in
        // the worker rewrites w^l, which the chain still reads on its way to delta^{l-1}: layer l's work then
        // starts once delta^{l-1} is there (layer 2's, whose weights the chain never reads, with delta^2).
        if (chain_only) continue;                       // the chain alone (a timing aid): no gradient is formed
        if (in_line) {
            if (!sgd || l == 2) st = enqueue_grads(net, l, s);
            if (st == LF_OK && sgd && l < L) st = enqueue_grads(net, l + 1, s);
            if (st != LF_OK) return st;
        } else {
            LF_HIP(net, hipEventRecord(net->ev_delta[l - 2], s));
            if (!sgd || l == 2) st = enqueue_grads_on_worker(net, l, k, nstreams, net->ev_delta[l - 2], used);
            if (st == LF_OK && sgd && l < L)
                st = enqueue_grads_on_worker(net, l + 1, k, nstreams, net->ev_delta[l - 2], used);
            if (st != LF_OK) return st;
        }
    }
    if (!in_line && !chain_only) {   // join
        for (int j = 0; j < nstreams; ++j) {
            if (!used[j]) continue;
            LF_HIP(net, hipEventRecord(net->ev_done[j], net->workers[j]));
            LF_HIP(net, hipStreamWaitEvent(s, net->ev_done[j], 0));
        }
    }
    net->bwd_done = !chain_only;
    if (sgd) net->stepped = true;                      // the stored activations belong to the old weights
    return LF_OK;
}

// Address of this device's copy of `scratch` (asked once per device, with that device current).
lf_status static_scratch_of_current_device(lf_net* net, void** out) {
    int dev = -1;
    LF_HIP(net, hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices)
        return fail(net, LF_EUNSUPPORTED, "lf_backward_leapfrog_noalloc: device index beyond 63");
    std::lock_guard<std::mutex> lock(g_static_scratch_mutex);
    if (!g_static_scratch[dev]) {
        void* p = nullptr;
        LF_HIP(net, hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return fail(net, LF_EHIP, "lf_backward_leapfrog_noalloc: the static scratch has no device address");
        g_static_scratch[dev] = p;
    }
    *out = g_static_scratch[dev];
    return LF_OK;
}

}  // namespace

extern "C" {

size_t lf_workspace_bytes_widths(int L, const int* n, int B, lf_dtype dt) {
    if (!valid_shape(L, n, B, dt)) return 0;
    const size_t t = make_layout(L, n, B, dt).total;
    return t ? t : kAlign;
}

size_t lf_workspace_bytes(int L, int N, int B, lf_dtype dt) {
    if (L < 2 || L > kMaxL) return 0;
    const std::vector<int> n((size_t)L, N);
    return lf_workspace_bytes_widths(L, n.data(), B, dt);
}

lf_status lf_create_widths(lf_net** out, int L, const int* n, int B, lf_dtype dt, lf_cost cost, void* workspace,
                           size_t workspace_bytes) {
    if (!out) return fail(nullptr, LF_EINVAL, "lf_create: out is NULL");
    *out = nullptr;
    if (!valid_shape(L, n, B, dt))
        return fail(nullptr, LF_EINVAL,
                    "lf_create: need 2 <= L <= 4096, B >= 1, every width a positive multiple of 4 (fp32) or 8 (bf16)");
    if (cost != LF_COST_QUADRATIC) return fail(nullptr, LF_EINVAL, "lf_create: unknown cost");
    if (!workspace) return fail(nullptr, LF_EINVAL, "lf_create: workspace is NULL");
    if (reinterpret_cast<uintptr_t>(workspace) % kAlign)
        return fail(nullptr, LF_EINVAL, "lf_create: workspace must be 256-byte aligned");
    if (workspace_bytes < lf_workspace_bytes_widths(L, n, B, dt))
        return fail(nullptr, LF_EINVAL, "lf_create: workspace smaller than lf_workspace_bytes()");
    lf_net* net = new (std::nothrow) lf_net();
    if (!net) return fail(nullptr, LF_ENOMEM, "lf_create: out of host memory");
    const int N = widest(L, n);
    net->L = L; net->N = N; net->B = B; net->dt = dt; net->cost = cost;
    net->uniform = all_equal(L, n);
    net->inner_uniform = inner_layers_equal(L, n);
    net->sched = LF_SCHED_AUTO;
    net->cost_scale = 1.0f;
    net->sgd_eta = 0.0f;
    net->ws = static_cast<char*>(workspace);
    net->lay = make_layout(L, n, B, dt);
    net->x1 = nullptr;
    net->have_params = net->have_grads = net->fwd_done = net->bwd_done = net->stepped = false;
    net->have_master = false;
    net->gemm = lf::gemm_plan(N, B, dt == LF_BF16);
    net->debug_flags = 0; net->p_failed_over = false; net->p_fused_ok = false;
    net->p_ready = false; net->p_tables_dirty = true; net->p_groups = net->p_rpg = net->p_bgroups = net->p_tpr = 0; net->p_workers = 0;
    net->p_abort_host = nullptr; net->p_abort_dev_view = nullptr;
    net->err = "no error";
    try {
        net->n.assign(n, n + L);
        net->w.assign(L - 1, nullptr); net->b.assign(L - 1, nullptr);
        net->gw.assign(L - 1, nullptr); net->gb.assign(L - 1, nullptr);
        net->w32.assign(L - 1, nullptr);
    } catch (...) {
        delete net;
        return fail(nullptr, LF_ENOMEM, "lf_create: out of host memory");
    }
    *out = net;
    return LF_OK;
}

lf_status lf_create(lf_net** out, int L, int N, int B, lf_dtype dt, lf_cost cost, void* workspace,
                    size_t workspace_bytes) {
    if (out) *out = nullptr;
    if (L < 2 || L > kMaxL)
        return fail(nullptr, LF_EINVAL,
                    "lf_create: need 2 <= L <= 4096, B >= 1, N a positive multiple of 4 (fp32) or 8 (bf16)");
    std::vector<int> n;
    try {
        n.assign((size_t)L, N);
    } catch (...) {
        return fail(nullptr, LF_ENOMEM, "lf_create: out of host memory");
    }
    return lf_create_widths(out, L, n.data(), B, dt, cost, workspace, workspace_bytes);
}

lf_status lf_set_params(lf_net* net, const void* const* w, const void* const* b) {
    if (!net) return LF_EINVAL;
    if (!w || !b) return fail(net, LF_EINVAL, "lf_set_params: NULL pointer array");
    for (int i = 0; i < net->L - 1; ++i) {
        if (!w[i] || !b[i]) return fail(net, LF_EINVAL, "lf_set_params: NULL layer pointer");
        if (!aligned16(w[i]) || !aligned16(b[i]))
            return fail(net, LF_EINVAL, "lf_set_params: pointers must be 16-byte aligned");
    }
    for (int i = 0; i < net->L - 1; ++i) { net->w[i] = w[i]; net->b[i] = static_cast<const float*>(b[i]); }
    net->have_params = true;
    net->p_tables_dirty = true;
    net->fwd_done = net->bwd_done = false;
    return LF_OK;
}

lf_status lf_set_grad_buffers(lf_net* net, float* const* nabla_w, float* const* nabla_b) {
    if (!net) return LF_EINVAL;
    if (!nabla_w || !nabla_b) return fail(net, LF_EINVAL, "lf_set_grad_buffers: NULL pointer array");
    for (int i = 0; i < net->L - 1; ++i) {
        if (!nabla_w[i] || !nabla_b[i]) return fail(net, LF_EINVAL, "lf_set_grad_buffers: NULL layer pointer");
        if (!aligned16(nabla_w[i]) || !aligned16(nabla_b[i]))
            return fail(net, LF_EINVAL, "lf_set_grad_buffers: pointers must be 16-byte aligned");
    }
    for (int i = 0; i < net->L - 1; ++i) { net->gw[i] = nabla_w[i]; net->gb[i] = nabla_b[i]; }
    net->have_grads = true;
    net->p_tables_dirty = true;
    net->bwd_done = false;
    return LF_OK;
}

lf_status lf_set_schedule(lf_net* net, lf_sched sched) {
    if (!net) return LF_EINVAL;
    switch (sched) {
        case LF_SCHED_AUTO:
        case LF_SCHED_STREAMS:
            net->sched = sched;
            return LF_OK;
        case LF_SCHED_REDUNDANT:
            if (!single_sample_path(net->N, net->B, net->dt))
                return fail(net, LF_EUNSUPPORTED, "lf_set_schedule: Algorithm 1 as printed runs for B = 1, fp32, N <= 16384");
            net->sched = sched;
            return LF_OK;
        case LF_SCHED_PERSISTENT:
        case LF_SCHED_FUSED:
            if (!persistent_possible(net))
                return fail(net, LF_EUNSUPPORTED,
                            "lf_set_schedule: the persistent kernels need B = 1, fp32, L <= 1025, layers 2..L-1 of one width N <= 4096, "
                            "the first and the last layer no wider");
            net->sched = sched;
            return LF_OK;
        default:
            return fail(net, LF_EINVAL, "lf_set_schedule: unknown schedule");
    }
}

lf_status lf_set_debug_flags(lf_net* net, unsigned flags) {
    if (!net) return LF_EINVAL;
    if (flags & ~(unsigned)LF_DEBUG_CHAIN_ONLY) return fail(net, LF_EINVAL, "lf_set_debug_flags: unknown flag");
    net->debug_flags = flags;
    net->bwd_done = false;
    return LF_OK;
}

lf_status lf_set_cost_scale(lf_net* net, int log2_scale) {
    if (!net) return LF_EINVAL;
    if (log2_scale < -126 || log2_scale > 127)
        return fail(net, LF_EINVAL, "lf_set_cost_scale: need -126 <= log2_scale <= 127");
    net->cost_scale = std::ldexp(1.0f, log2_scale);
    return LF_OK;
}

lf_status lf_set_master_weights(lf_net* net, float* const* w32) {
    if (!net) return LF_EINVAL;
    if (net->dt != LF_BF16)
        return fail(net, LF_EINVAL, "lf_set_master_weights: fp32 weights are stepped in place; masters belong to bf16 nets");
    if (!w32) return fail(net, LF_EINVAL, "lf_set_master_weights: NULL pointer array");
    for (int i = 0; i < net->L - 1; ++i) {
        if (!w32[i]) return fail(net, LF_EINVAL, "lf_set_master_weights: NULL layer pointer");
        if (!aligned16(w32[i])) return fail(net, LF_EINVAL, "lf_set_master_weights: pointers must be 16-byte aligned");
    }
    for (int i = 0; i < net->L - 1; ++i) net->w32[i] = w32[i];
    net->have_master = true;
    return LF_OK;
}

lf_status lf_set_sgd(lf_net* net, float eta) {
    if (!net) return LF_EINVAL;
    if (!(eta >= 0.0f) || !std::isfinite(eta)) return fail(net, LF_EINVAL, "lf_set_sgd: need a finite eta >= 0");
    net->sgd_eta = eta;
    net->bwd_done = false;
    return LF_OK;
}

lf_status lf_forward(lf_net* net, const void* x1, void* hip_stream) {
    if (!net) return LF_EINVAL;
    if (!x1) return fail(net, LF_EINVAL, "lf_forward: x1 is NULL");
    if (!aligned16(x1)) return fail(net, LF_EINVAL, "lf_forward: x1 must be 16-byte aligned");
    if (!net->have_params) return fail(net, LF_ESTATE, "lf_forward: call lf_set_params first");
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    lf_status st0 = check_abort(net);
    if (st0 != LF_OK) return st0;
    net->x1 = x1;
    net->fwd_done = false;
    net->bwd_done = false;
    net->stepped = false;
    const bool bf = net->dt == LF_BF16;
    if (use_persistent(net)) {
        st0 = prepare_persistent(net, s);
        if (st0 != LF_OK) return st0;
        lf::PersistArgs A = persist_args(net, nullptr, 1);
        A.nap = net->p_nap_fwd;
        LF_HIP(net, lf::launch_fwd_persistent(A, s));
        net->fwd_done = true;
        return LF_OK;
    }
    for (int l = 2; l <= net->L; ++l) {
        if (single_sample_path(net->N, net->B, net->dt)) {
            LF_HIP(net, lf::launch_fwd_gemv_f32(static_cast<const float*>(net->w[l - 2]), net->b[l - 2],
                                                static_cast<const float*>(net->a_ptr(l - 1)),
                                                static_cast<float*>(net->a_ptr(l)), net->width(l),
                                                net->width(l - 1), s));
        } else {
            LF_HIP(net, lf::launch_fwd_gemm(net->w[l - 2], net->b[l - 2], net->a_ptr(l - 1), net->a_ptr(l),
                                            net->raw(), net->width(l), net->width(l - 1), net->B, bf,
                                            net->gemm, s));
        }
    }
    net->fwd_done = true;
    return LF_OK;
}

lf_status lf_backward_leapfrog(lf_net* net, const void* y, int k, void* hip_stream) {
    if (!net) return LF_EINVAL;
    lf_status st = check_backward_call(net, y, k);
    if (st != LF_OK) return st;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    net->bwd_done = false;
    st = check_abort(net);
    if (st != LF_OK) return st;
    const bool chain_only = (net->debug_flags & LF_DEBUG_CHAIN_ONLY) != 0;
    if (chain_only && net->sched == LF_SCHED_REDUNDANT)
        return fail(net, LF_EUNSUPPORTED, "lf_backward_leapfrog: LF_DEBUG_CHAIN_ONLY has no meaning for LF_SCHED_REDUNDANT");
    if (use_persistent(net)) {
        if (net->sched == LF_SCHED_FUSED && net->sgd_eta != 0.0f)
            return fail(net, LF_EUNSUPPORTED, "lf_backward_leapfrog: LF_SCHED_FUSED does not take the descent step");
        st = prepare_persistent(net, s);
        if (st != LF_OK) return st;
        if (net->sched == LF_SCHED_FUSED && !net->p_fused_ok)
            return fail(net, LF_EUNSUPPORTED, "lf_backward_leapfrog: the device cannot hold the fused kernel's workgroups at once");
        lf::PersistArgs A = persist_args(net, y, k);
        A.nap = net->p_nap_bwd;
        LF_HIP(net, lf::launch_bwd_persistent(A, s));
        net->bwd_done = !chain_only;
        if (net->sgd_eta != 0.0f) net->stepped = true;
        return LF_OK;
    }
    if (net->sched == LF_SCHED_REDUNDANT) {
        st = backward_redundant(net, y, k, s);
        if (st == LF_OK) net->bwd_done = true;
        return st;
    }
    st = ensure_workers(net, k);
    if (st != LF_OK) return st;
    return backward_streams(net, y, k, s, net->partial(), net->raw(), /*in_line=*/k == 1);
}

size_t lf_noalloc_scratch_limit(void) { return LF_STATIC_SCRATCH_BYTES; }

lf_status lf_backward_leapfrog_noalloc(lf_net* net, const void* y, int k, void* hip_stream) {
    if (!net) return LF_EINVAL;
    lf_status st = check_backward_call(net, y, k);
    if (st != LF_OK) return st;
    if (net->sched == LF_SCHED_REDUNDANT || net->sched == LF_SCHED_FUSED)
        return fail(net, LF_EUNSUPPORTED, "lf_backward_leapfrog_noalloc: runs the stream schedule's kernels only");
    // what the chain products of this net really use: the single-sample row-block partial sums, or the split-K
    // partials under the net's plan (the workspace reserves room for the deepest split any plan could take)
    size_t need = net->lay.partial_bytes;
    if (!single_sample_path(net->N, net->B, net->dt))
        for (int l = 2; l < net->L; ++l)
            need = std::max(need, 4 * lf::split_scratch_floats(net->width(l), net->width(l + 1), net->B,
                                                               net->dt == LF_BF16, net->gemm, true));
    if (need > LF_STATIC_SCRATCH_BYTES)
        return fail(net, LF_EUNSUPPORTED,
                    "lf_backward_leapfrog_noalloc: this shape needs " + std::to_string(need) +
                        " bytes of chain scratch, the static scratch holds " + std::to_string(LF_STATIC_SCRATCH_BYTES));
    void* area = nullptr;
    st = static_scratch_of_current_device(net, &area);
    if (st != LF_OK) return st;
    net->bwd_done = false;
    // every word of the scratch a pass reads it has written before (the chain's partial sums are stored
    // whole, then summed): nothing needs clearing between calls
    return backward_streams(net, y, k, static_cast<hipStream_t>(hip_stream), static_cast<float*>(area),
                            static_cast<float*>(area), /*in_line=*/true);
}

lf_status lf_grads(lf_net* net, int l, const float** nabla_w, const float** nabla_b) {
    if (!net) return LF_EINVAL;
    if (l < 2 || l > net->L) return fail(net, LF_EINVAL, "lf_grads: layer index must be in 2..L");
    if (!net->bwd_done) return fail(net, LF_ESTATE, "lf_grads: no backward pass has been enqueued");
    if (net->sgd_eta != 0.0f)
        return fail(net, LF_ESTATE, "lf_grads: with lf_set_sgd the gradients are applied, not stored");
    const lf_status st = check_abort(net);
    if (st != LF_OK) return st;
    if (nabla_w) *nabla_w = net->gw[l - 2];
    if (nabla_b) *nabla_b = net->gb[l - 2];
    return LF_OK;
}

lf_status lf_activations(lf_net* net, int l, const void** a_l, const float** delta_l) {
    if (!net) return LF_EINVAL;
    if (l < 1 || l > net->L) return fail(net, LF_EINVAL, "lf_activations: layer index must be in 1..L");
    if (!net->fwd_done) return fail(net, LF_ESTATE, "lf_activations: no forward pass has been enqueued");
    if (a_l) *a_l = net->a_ptr(l);
    if (delta_l) *delta_l = l >= 2 ? net->d_ptr(l) : nullptr;
    return LF_OK;
}

int lf_schedule_worker(int L, int k, int l) {
    if (L < 2 || k < 1 || k > L - 1 || l < 2 || l > L) return -1;
    return (L - l) % k;
}

int lf_algorithm1_owner(int L, int k, int l) {
    if (L < 2 || k < 1 || k > L - 1 || l < 2 || l > L) return -1;
    return l > L - k ? k : (L - l) % k;
}

const char* lf_last_error(const lf_net* net) { return net ? net->err.c_str() : g_create_error.c_str(); }

void lf_destroy(lf_net* net) {
    if (!net) return;
    for (hipStream_t s : net->workers) (void)hipStreamDestroy(s);
    for (hipEvent_t e : net->ev_delta) (void)hipEventDestroy(e);
    for (hipEvent_t e : net->ev_done) (void)hipEventDestroy(e);
    if (net->p_abort_host) (void)hipHostFree(net->p_abort_host);
    delete net;
}

}  // extern "C"
