// C-ABI entry points of the compression-step library (see include/condensa.h): argument checks,
// table building, workspace carving and the kernel launch sequences.
#include <memory>

#include "host.h"
#include "k_apply.h"
#include "k_quantize.h"
#include "k_fused.h"
#include "k_select.h"
#include "k_small.h"
#include "k_structure.h"
#include "k_window.h"
#include "k_struct_fused.h"
#include "k_struct_list.h"

namespace condensa {

std::atomic<int> g_last_hip_error{0};
std::atomic<uint64_t> g_launches{0};

// ---- configuration ---------------------------------------------------------------------------------

namespace {
// process-wide defaults: what a NULL condensa_config stands for
std::atomic<int64_t> g_options[CONDENSA_OPT_COUNT] = {{0}, {0}, {80}, {0}, {0}, {0}, {0}};

bool option_value_ok(int option, int64_t value) {
    if (value < 0) return false;
    switch (option) {
        case CONDENSA_OPT_SELECT_PATH:   return value <= 2;
        case CONDENSA_OPT_SAMPLE_LOG2:   return value == 0 || (value >= 10 && value <= 26);
        case CONDENSA_OPT_WINDOW_MARGIN: return value <= 0x7FFFFFFF;
        case CONDENSA_OPT_CAND_SHIFT:    return value <= 30;
        case CONDENSA_OPT_PROFILE:       return value < (1 << CONDENSA_PHASE_COUNT);
        case CONDENSA_OPT_APPLY_THREADS: return value == 0 || value == 64 || value == 128 || value == 256;
        case CONDENSA_OPT_FUSED_SWEEP:   return value <= 1;
        default: return false;
    }
}
}  // namespace

condensa_status set_default_option(int option, int64_t value) {
    if (!option_value_ok(option, value)) return CONDENSA_ERR_ARG;
    g_options[option].store(value);
    return CONDENSA_OK;
}

condensa_status resolve_config(const condensa_config* c, Config* out) {
    if (c == nullptr) {
        for (int i = 0; i < CONDENSA_OPT_COUNT; ++i) out->v[i] = g_options[i].load();
        return CONDENSA_OK;
    }
    if (c->reserved != 0) return CONDENSA_ERR_ARG;
    const int64_t v[CONDENSA_OPT_COUNT] = {c->select_path, c->sample_log2, c->window_margin, c->cand_shift,
                                           c->profile, c->apply_threads, c->fused_sweep};
    for (int i = 0; i < CONDENSA_OPT_COUNT; ++i) {
        if (!option_value_ok(i, v[i])) return CONDENSA_ERR_ARG;
        out->v[i] = v[i];
    }
    return CONDENSA_OK;
}

// ---- pinned staging ring -------------------------------------------------------------------------

namespace {
struct Stage {
    void* host = nullptr;
    size_t cap = 0;
    hipEvent_t ev = nullptr;
    bool pending = false;
};
constexpr int kRing = 8;
Stage g_ring[kRing];
int g_ring_next = 0;
std::mutex g_ring_mu;
}  // namespace

condensa_status stage_upload(void* dst_dev, const void* src_host, size_t bytes, hipStream_t stream) {
    if (bytes == 0) return CONDENSA_OK;
    std::lock_guard<std::mutex> lock(g_ring_mu);
    Stage& s = g_ring[g_ring_next];
    g_ring_next = (g_ring_next + 1) % kRing;
    if (s.pending) {
        CONDENSA_HIP(hipEventSynchronize(s.ev));
        s.pending = false;
    }
    if (s.cap < bytes) {
        if (s.host) CONDENSA_HIP(hipHostFree(s.host));
        s.host = nullptr;
        s.cap = 0;
        const size_t cap = align_up(bytes < (64u << 10) ? (64u << 10) : bytes, 4096);
        CONDENSA_HIP(hipHostMalloc(&s.host, cap, hipHostMallocDefault));
        s.cap = cap;
    }
    if (!s.ev) CONDENSA_HIP(hipEventCreateWithFlags(&s.ev, hipEventDisableTiming));
    std::memcpy(s.host, src_host, bytes);
    CONDENSA_HIP(hipMemcpyAsync(dst_dev, s.host, bytes, hipMemcpyHostToDevice, stream));
    CONDENSA_HIP(hipEventRecord(s.ev, stream));
    s.pending = true;
    return CONDENSA_OK;
}

// ---- phase timing ----------------------------------------------------------------------------------

namespace {
struct Interval {
    hipEvent_t a = nullptr, b = nullptr;
    int phase = 0;
};
std::vector<Interval> g_intervals;          // both events recorded, not yet read
std::vector<hipEvent_t> g_event_pool;
double g_phase_ms[CONDENSA_PHASE_COUNT] = {};
u64 g_phase_n[CONDENSA_PHASE_COUNT] = {};
std::mutex g_prof_mu;

hipEvent_t take_event() {                   // g_prof_mu held
    if (!g_event_pool.empty()) {
        hipEvent_t e = g_event_pool.back();
        g_event_pool.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}
}  // namespace

PhaseTimer::PhaseTimer(int phase, hipStream_t stream, const Config& cfg) : phase_(phase), stream_(stream) {
    if (((cfg[CONDENSA_OPT_PROFILE] >> phase) & 1) == 0) return;
    hipEvent_t a, b;
    {
        std::lock_guard<std::mutex> lock(g_prof_mu);
        a = take_event();
        b = take_event();
    }
    if (a && b && hipEventRecord(a, stream_) == hipSuccess) {
        a_ = a;
        b_ = b;
        return;
    }
    std::lock_guard<std::mutex> lock(g_prof_mu);
    if (a) g_event_pool.push_back(a);
    if (b) g_event_pool.push_back(b);
}

PhaseTimer::~PhaseTimer() {
    if (!a_) return;
    const bool ok = hipEventRecord(b_, stream_) == hipSuccess;
    std::lock_guard<std::mutex> lock(g_prof_mu);
    if (ok) {
        Interval iv;
        iv.a = a_; iv.b = b_; iv.phase = phase_;
        g_intervals.push_back(iv);
    } else {
        g_event_pool.push_back(a_);
        g_event_pool.push_back(b_);
    }
}

// ---- workspace layout ----------------------------------------------------------------------------

static u64 window_sample_size(u64 N, const Config& cfg) {
    const int64_t opt = cfg[CONDENSA_OPT_SAMPLE_LOG2];
    u64 s;
    if (opt > 0) s = static_cast<u64>(1) << (opt > 26 ? 26 : opt);
    else {
        s = N / 8;
        if (s < (1u << 18)) s = 1u << 18;
        if (s > (1u << 21)) s = 1u << 21;
    }
    s = (s + kSampleUnit - 1) / kSampleUnit * kSampleUnit;
    return s;
}

static u64 window_cand_capacity(u64 N, int J, const Config& cfg) {
    const int64_t opt = cfg[CONDENSA_OPT_CAND_SHIFT];
    const int shift = (opt > 0 && opt < 40) ? static_cast<int>(opt) : (J > 1 ? 3 : 5);
    u64 c = N >> shift;
    if (c < 4096) c = 4096;
    return c;
}

Layout make_layout(int op, u64 N, u64 F, int n_tensors, int J, int scope, const Config& cfg, bool no_window) {
    Layout L;
    const bool per_tensor = (scope == CONDENSA_SCOPE_PER_TENSOR);
    const bool structure = (op == CONDENSA_OP_FILTER_PRUNE || op == CONDENSA_OP_BLOCK_PRUNE);
    if (structure || op == CONDENSA_OP_LC_STEP) J = 1;
    L.n_groups = per_tensor ? (n_tensors > 0 ? n_tensors : 1) : 1;
    L.n_slots = L.n_groups * J;
    L.max_chunks = N / kChunk + static_cast<u64>(n_tensors);
    L.max_schunks = F / kChunk + static_cast<u64>(n_tensors);
    size_t off = 0;
    L.td = off;     off += align_up(static_cast<size_t>(n_tensors + 1) * sizeof(TensorDesc));
    L.out = off;    off += align_up(static_cast<size_t>(J) * (n_tensors > 0 ? n_tensors : 1) * sizeof(OutDesc));
    L.slots = off;  off += align_up(static_cast<size_t>(L.n_slots) * sizeof(Slot) + (structure ? 3 : 2 * kMaxJ) * sizeof(Slot));
    L.upload_bytes = off;
    L.zero_begin = off;
    L.ctl = off;    off += align_up(sizeof(Control));
    L.hist0 = off;  off += align_up(static_cast<size_t>(L.n_groups) * kBins * sizeof(u64));
    // later-level histograms of the rankings over the data (one per ranking and level under GLOBAL scope),
    // then the window path's: candidate rankings [3][J], the sample's boundary rankings [2][2J + 1] and its
    // shared level 0 (see make_window_args)
    size_t n_hx = 2u * static_cast<size_t>(L.n_slots);
    if (!structure && !per_tensor) n_hx += 3u * J + 2u * (2u * J + 1u) + 1u;
    // structures under GLOBAL scope: one histogram per level of the 63-bit ranking, then (one-sweep block pruning) the
    // block sample's boundary rankings [2][3] and their shared level 0
    if (structure && !per_tensor) n_hx = kStructLevels + 2u * 3u + 1u;
    L.histx = off;  off += align_up(n_hx * kBins * sizeof(u64));
    // coarse sums of every histogram from hist0 on (the two regions above are contiguous: their sizes are multiples of 16 KB)
    L.histc = off;  off += align_up((static_cast<size_t>(L.n_groups) + n_hx) * kCoarse * sizeof(u64));
    if (!structure && !per_tensor) { L.seg = off; off += align_up(static_cast<size_t>(kSegs) * (2 + kMaxJ) * sizeof(u64)); }
    if (structure && !per_tensor) { L.seg = off; off += align_up(static_cast<size_t>(kSegs) * 2 * sizeof(u64)); }
    // per-chunk tie counts and the flags of the chunks that can hold ties: cleared with the counters, because the
    // tie search only visits flagged chunks and leaves the others' counts alone
    const u64 tie_chunks = structure ? L.max_schunks : ((op == CONDENSA_OP_COUNT_NONZERO || op == CONDENSA_OP_LC_SGD_STEP) ? 0 : L.max_chunks);
    L.tiecnt = off; off += align_up(static_cast<size_t>(J) * tie_chunks * sizeof(u32));
    if (!structure) { L.tiehit = off; off += align_up(static_cast<size_t>(tie_chunks + 1) * sizeof(u32)); }
    const bool tie_lists = !structure && !per_tensor && tie_chunks > 0;
    if (tie_lists) { L.tl_cnt = off; off += align_up(static_cast<size_t>(kMaxJ) * sizeof(u64)); }
    L.zero_bytes = off - L.zero_begin;
    L.chunk_map = off; off += align_up(static_cast<size_t>(L.max_chunks + 1) * sizeof(u32));
    if (tie_lists) {
        // small calls on the automatic path finish on one list that can hold every element (k_small.h)
        if (!no_window && N > 0 && N <= kSmallCallElems && cfg[CONDENSA_OPT_SELECT_PATH] == 0) L.small_cap = N;
        u64 entries = static_cast<u64>(J) * kTieListCap;
        if (entries < L.small_cap) entries = L.small_cap;
        L.tl_key = off; off += align_up(static_cast<size_t>(entries) * sizeof(u32));
        L.tl_idx = off; off += align_up(static_cast<size_t>(entries) * sizeof(u64));
    }
    if (structure) {
        L.skeys = off;  off += align_up(static_cast<size_t>(F) * sizeof(u64));
        L.sblock = off; off += align_up(static_cast<size_t>(F / kBlock + 2) * sizeof(u32));
        L.smask = off;  off += align_up(static_cast<size_t>(F) + 1);
        if (!per_tensor) {                                  // one-sweep block pruning: sample keys and the list of window blocks
            u64 sc = F / 8;
            sc = sc < (1u << 12) ? (1u << 12) : (sc > (1u << 17) ? (1u << 17) : sc);
            L.sample_cap = sc;
            // room for an eighth of the blocks, and for all of them while that costs under a megabyte
            L.cand_cap = F / 8;
            if (L.cand_cap < (1u << 16)) L.cand_cap = F < (1u << 16) ? (F < 4096 ? 4096 : F) : (1u << 16);
            if (F <= kSmallCallElems && L.cand_cap < F) L.cand_cap = F;   // the list of k_struct_list.h holds every structure
            L.sample = off;   off += align_up(L.sample_cap * sizeof(u32));
            L.cand_key = off; off += align_up(L.cand_cap * sizeof(u32));      // ids of the listed blocks
            L.cand_idx = off; off += align_up(L.cand_cap * sizeof(u64));      // their aggregate keys
        }
    } else if (!per_tensor && !no_window && op != CONDENSA_OP_COUNT_NONZERO && op != CONDENSA_OP_LC_SGD_STEP) {
        L.sample_cap = window_sample_size(N, cfg);
        L.cand_cap = window_cand_capacity(N, J, cfg);
        L.sample = off;   off += align_up(L.sample_cap * sizeof(u32));
        L.cand_key = off; off += align_up(L.cand_cap * sizeof(u32));
        L.cand_idx = off; off += align_up(L.cand_cap * sizeof(u64));
        L.sorted_windows = off; off += align_up(256);             // SortedWindows (196 B)
        if (J == 1) {
            L.cand_w = off;   off += align_up(L.cand_cap * sizeof(float));
            L.cand_lam = off; off += align_up(L.cand_cap * sizeof(float));
        }
    }
    L.total = off;
    return L;
}

// ---- tables ---------------------------------------------------------------------------------------

// Host memory of one call's tables.  The usual entry points take it from the heap; the entry point for
// callers that cannot allocate hands out pieces of a fixed buffer on its own stack instead.
class HostArena {
public:
    HostArena() = default;                                         // heap
    HostArena(char* fixed, size_t bytes) : fixed_(fixed), left_(bytes) {}
    HostArena(const HostArena&) = delete;
    HostArena& operator=(const HostArena&) = delete;
    // n zero-initialised objects of T (trivially copyable table types), or nullptr when a fixed buffer is used up
    template <typename T>
    T* array(size_t n) {
        const size_t bytes = align_up((n ? n : 1) * sizeof(T), 64);
        char* p;
        if (fixed_) {
            if (bytes > left_) return nullptr;
            p = fixed_;
            fixed_ += bytes;
            left_ -= bytes;
        } else {
            heap_.emplace_back(new char[bytes]);
            p = heap_.back().get();
        }
        std::memset(p, 0, bytes);
        return reinterpret_cast<T*>(p);
    }
private:
    char* fixed_ = nullptr;
    size_t left_ = 0;
    std::vector<std::unique_ptr<char[]>> heap_;
};

struct Tables {
    TensorDesc* td = nullptr;        // n_tensors + 1 (sentinel)
    int n_td = 0;
    u64 N = 0, n_chunks = 0, F = 0, n_schunks = 0;
    bool vec = true;
};

static condensa_status build_tensor_table(const condensa_tensor* tensors, int n_tensors, Tables* tb, HostArena& arena) {
    if (n_tensors < 0 || n_tensors > CONDENSA_MAX_TENSORS) return CONDENSA_ERR_SIZE;
    if (n_tensors > 0 && tensors == nullptr) return CONDENSA_ERR_NULL;
    tb->td = arena.array<TensorDesc>(static_cast<size_t>(n_tensors) + 1);
    if (tb->td == nullptr) return CONDENSA_ERR_SIZE;
    tb->n_td = n_tensors + 1;
    u64 flat = 0, chunk = 0;
    for (int t = 0; t < n_tensors; ++t) {
        u64 n;
        if (!tensor_elems(tensors[t], &n)) return CONDENSA_ERR_SHAPE;
        if (n > 0 && tensors[t].w == nullptr) return CONDENSA_ERR_NULL;
        TensorDesc& d = tb->td[t];
        d.w = tensors[t].w;
        d.n = n;
        d.flat_start = flat;
        d.chunk_start = chunk;
        flat += n;
        if (flat > kMaxElems) return CONDENSA_ERR_SIZE;
        chunk += (n + kChunk - 1) / kChunk;
        if (n > 0 && !aligned16(d.w)) tb->vec = false;
    }
    TensorDesc& end = tb->td[n_tensors];
    end.flat_start = flat;
    end.chunk_start = chunk;
    tb->N = flat;
    tb->n_chunks = chunk;
    return CONDENSA_OK;
}

static condensa_status check_workspace(const void* ws, size_t bytes, const Layout& L) {
    if (ws == nullptr) return CONDENSA_ERR_WORKSPACE;
    if (reinterpret_cast<uintptr_t>(ws) & 255u) return CONDENSA_ERR_WORKSPACE;
    if (bytes < L.total) return CONDENSA_ERR_WORKSPACE;
    return CONDENSA_OK;
}

static void init_slot(Slot* s, u64 n, u64 k, u32 path) {
    std::memset(s, 0, sizeof(Slot));
    s->n = n;
    s->k = k;
    s->path = path;
    if (k == 0) {
        s->state = kInactive;
        s->prefix = ~static_cast<u64>(0);
        s->remaining = 0;
        s->tie_end = 0;
    } else {
        s->state = kSelecting;
        s->prefix = 0;
        s->remaining = k;
        s->tie_end = n;
    }
}

// One density on the window path: the three rankings of the sample that bound (kRankHi, kRankLo) and estimate
// (kRankMid) the threshold of `main`.  Their ranks depend on the number of valid sample keys, which only the
// device knows, so the host passes the rule and the device turns it into a rank (sample_rank).
static void init_sample_slots(Slot* three, const Slot& main, int64_t margin16) {
    for (u32 i = 0; i < 3; ++i) {
        Slot& s = three[i];
        std::memset(&s, 0, sizeof(Slot));
        s.rank_rule = kRankHi + i;
        s.margin16 = static_cast<u32>(margin16);
        s.p = main.n ? static_cast<double>(main.k) / static_cast<double>(main.n) : 0.0;
        s.hi = 0x7FFFFFFFu;                                     // every valid sample key takes part
        s.state = main.state == kSelecting ? kSelecting : kDone;
        s.prefix = (s.rank_rule == kRankHi && s.state == kDone) ? 0x7FFFFFFFu : 0u;
    }
}

template <typename T>
static T* at(void* ws, size_t off) { return reinterpret_cast<T*>(static_cast<char*>(ws) + off); }

static unsigned fill_grid(u64 words) {
    u64 b = (words + kBlock - 1) / kBlock;
    if (b > 4096) b = 4096;
    if (b == 0) b = 1;
    return static_cast<unsigned>(b);
}

// Radix levels over the weights: 3 x (histogram sweep + bin search).
template <bool LC, bool VEC>
static condensa_status launch_radix_levels(const DataArgs& a, int n_slots, hipStream_t st, const Config& cfg,
                                           int levels = n_levels(31)) {
    if (a.n_chunks > 0) {
        // as the gated fallback of the window path these launches are (normally empty) resolve work
        PhaseTimer timer(a.only_failed ? CONDENSA_PHASE_RESOLVE : CONDENSA_PHASE_SWEEP, st, cfg);
        for (int level = 0; level < levels; ++level) {
            // Every workgroup flushes the non-zero bins of its LDS histograms (J of them past level 0) with
            // global atomics: few wide workgroups keep that flush small (level 0 of 20 M weights: 36 -> 19 us).
            const bool wide = !a.per_tensor;
            const unsigned threads = wide ? 1024 : kBlock;
            // measured: best of 128..1024 workgroups at 1.2 G weights; on 20 M weights (10 rankings) 256 x 1024
            // threads take 192 us per call against 221 (512 x 512), 275 (512 x 256) and 351 (1024 x 256)
            const u64 cap = wide ? 256 : 2048;
            const u64 per_iter = threads / kBlock;
            u64 blocks = (a.n_chunks + per_iter - 1) / per_iter;
            if (blocks > cap) blocks = cap;
            u64 cpb = (a.n_chunks + blocks - 1) / blocks;
            cpb = (cpb + per_iter - 1) / per_iter * per_iter;
            blocks = (a.n_chunks + cpb - 1) / cpb;
            const int nj = a.J < kSlotBatch ? a.J : kSlotBatch;
            const size_t lds = static_cast<size_t>(level == 0 ? kBins : nj * (1 << level_of(31, level).bits)) * sizeof(u32);
            hipLaunchKernelGGL((k_hist_data<LC, VEC>), dim3(static_cast<unsigned>(blocks)), dim3(threads), lds, st, a, level, cpb);
            CONDENSA_LAUNCH_CHECK();
            if (a.merged) continue;                            // the next kernel folds this level in itself
            hipLaunchKernelGGL(k_scan_level, dim3(n_slots), dim3(kBlock), 0, st, a.slots, a.hist0, a.histx, a.J, 31,
                               level, a.ctl, a.only_failed, &a.ctl->need_tie);
            CONDENSA_LAUNCH_CHECK();
        }
    }
    return CONDENSA_OK;
}

template <bool LC, bool VEC>
static condensa_status launch_ties_and_results(const DataArgs& a, int n_slots, int n_groups,
                                               condensa_select* results, hipStream_t st, const Config& cfg) {
    PhaseTimer timer(CONDENSA_PHASE_RESOLVE, st, cfg);
    if (a.n_chunks > 0) {
        // merged form: every workgroup first folds in the last level for each ranking, so fewer of them
        const u64 tie_cap = a.merged ? 1024 : 4096;
        const unsigned tie_blocks = static_cast<unsigned>(a.n_chunks < tie_cap ? a.n_chunks : tie_cap);
        hipLaunchKernelGGL((k_tie_count<LC, VEC>), dim3(tie_blocks), dim3(kBlock), 0, st, a);
        CONDENSA_LAUNCH_CHECK();
    }
    hipLaunchKernelGGL((k_tie_locate<LC, VEC>), dim3(n_slots), dim3(kBlock), 0, st, a, results, n_groups);
    CONDENSA_LAUNCH_CHECK();
    return CONDENSA_OK;
}

template <bool LC, bool VEC>
static condensa_status run_selection(DataArgs a, const Layout& L, void* ws, bool use_window, int n_slots,
                                     int n_groups, condensa_select* results, hipStream_t st, const Config& cfg,
                                     const FusedRequest* fused = nullptr) {
    condensa_status rc;
    if (use_window) {
        rc = a.J == 1 ? launch_window_path_single<LC, VEC>(a, L, ws, st, cfg, fused)
                      : launch_window_path<LC, VEC>(a, L, ws, st, cfg);
        if (rc != CONDENSA_OK) return rc;
        a.only_failed = 1;
    }
    if (!use_window && a.small_cap >= a.N && a.n_chunks > 0 && a.merged) {
        // a small call: level 0, then the keys of the thresholds' bins as a list, then one workgroup per ranking
        rc = launch_radix_levels<LC, VEC>(a, n_slots, st, cfg, 1);
        if (rc != CONDENSA_OK) return rc;
        PhaseTimer timer(CONDENSA_PHASE_RESOLVE, st, cfg);
        hipLaunchKernelGGL((k_small_collect<LC, VEC>), dim3(static_cast<unsigned>(a.n_chunks < 1024 ? a.n_chunks : 1024)), dim3(kBlock), 0, st, a);
        CONDENSA_LAUNCH_CHECK();
        hipLaunchKernelGGL(k_small_finish, dim3(n_slots), dim3(kSmallFinishThreads), 0, st, a, results, bits_for(a.N - 1));
        CONDENSA_LAUNCH_CHECK();
        return CONDENSA_OK;
    }
    rc = launch_radix_levels<LC, VEC>(a, n_slots, st, cfg);
    if (rc != CONDENSA_OK) return rc;
    return launch_ties_and_results<LC, VEC>(a, n_slots, n_groups, results, st, cfg);
}

// Sampled window or radix levels?  Measured (one MI355X, 2^24..2^30 weights, 1/4/10 densities): the radix
// levels cost three sweeps whatever the number of densities and ~50 us of fixed work; the window path
// costs one sweep, ~0.2 ms of small kernels, and candidate lists and a sweep that grow with the number
// of densities.  One density breaks even near 2^26 element reads, four near 2^27.5, ten near 2^30.
static bool want_window(u64 N, bool per_tensor, int J, bool lc, const Config& cfg) {
    if (per_tensor) return false;
    if ((N >> kCandTensorShift) != 0) return false;        // candidates carry their tensor above a 44-bit flat index
    const int64_t mode = cfg[CONDENSA_OPT_SELECT_PATH];
    if (mode == 1) return false;
    if (mode == 2) return N >= 1;
    u64 need = static_cast<u64>(J) << 26;
    if (J > 4) need = need * static_cast<u64>(J) / 4;
    return N * (lc ? 2u : 1u) >= need;
}

}  // namespace condensa

namespace condensa {

// ---- static scratch for callers that cannot allocate ---------------------------------------------------
// One array per device, resident until the process ends.  Host code never uses the array's name as an
// address: scratch_for_current_device() asks the runtime for the device address once per device.

constexpr size_t kScratchBytes = static_cast<size_t>(2) << 20;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

namespace {
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mu;
}  // namespace

static condensa_status scratch_for_current_device(void** out) {
    int dev = -1;
    CONDENSA_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return CONDENSA_ERR_ARG;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (g_scratch_ptr[dev] == nullptr) {
        void* p = nullptr;
        CONDENSA_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (p == nullptr) return CONDENSA_ERR_HIP;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return CONDENSA_OK;
}

// Writes host words into device memory as kernel arguments: no staging buffer, nothing to allocate.
struct PokeWords { u64 w[448]; };
__global__ __launch_bounds__(kBlock) void k_poke(u64* dst, PokeWords src, u32 n) {
    for (u32 i = threadIdx.x; i < n; i += kBlock) dst[i] = src.w[i];
}

static condensa_status poke_upload(void* dst_dev, const char* src_host, size_t bytes, hipStream_t st) {
    constexpr size_t kPiece = sizeof(PokeWords);
    for (size_t off = 0; off < bytes; off += kPiece) {
        const size_t n = bytes - off < kPiece ? bytes - off : kPiece;      // bytes is a multiple of 256
        PokeWords pw;
        std::memcpy(pw.w, src_host + off, n);
        hipLaunchKernelGGL(k_poke, dim3(1), dim3(kBlock), 0, st, reinterpret_cast<u64*>(static_cast<char*>(dst_dev) + off),
                           pw, static_cast<u32>(n / 8));
        CONDENSA_LAUNCH_CHECK();
    }
    return CONDENSA_OK;
}

// condensa_prune and its allocation-free form share everything but where the host tables live, how they
// reach the device and where the workspace comes from.
static condensa_status prune_impl(const condensa_tensor* tensors, int n_tensors, const double* densities,
                                  int n_densities, int scope, float* const* theta, uint16_t* const* theta_f16,
                                  uint8_t* const* mask, condensa_select* results_dev, void* workspace_dev,
                                  size_t workspace_bytes, void* stream, const Config& cfg, HostArena& arena,
                                  bool no_alloc) {
    if (n_densities < 1 || n_densities > CONDENSA_MAX_DENSITIES) return CONDENSA_ERR_SIZE;
    if (densities == nullptr || results_dev == nullptr) return CONDENSA_ERR_NULL;
    if (scope != CONDENSA_SCOPE_GLOBAL && scope != CONDENSA_SCOPE_PER_TENSOR) return CONDENSA_ERR_ARG;
    for (int j = 0; j < n_densities; ++j)
        if (!density_ok(densities[j])) return CONDENSA_ERR_DENSITY;
    Tables tb;
    condensa_status rc = build_tensor_table(tensors, n_tensors, &tb, arena);
    if (rc != CONDENSA_OK) return rc;
    const int J = n_densities;
    const bool per_tensor = (scope == CONDENSA_SCOPE_PER_TENSOR);
    if (per_tensor && n_tensors == 0) return CONDENSA_OK;
    // the allocation-free form keeps to the radix levels, whose workspace is small whatever the input
    const Layout L = make_layout(CONDENSA_OP_PRUNE, tb.N, 0, n_tensors, J, scope, cfg, no_alloc);

    // output table, overlap and alignment checks
    const bool any_out = theta || theta_f16 || mask;
    const size_t n_out = static_cast<size_t>(J) * (n_tensors > 0 ? n_tensors : 1);
    OutDesc* out = arena.array<OutDesc>(n_out);
    ByteRange* ranges = arena.array<ByteRange>(static_cast<size_t>(n_tensors) * (1 + 3 * J) + 2);
    if (!out || !ranges) return CONDENSA_ERR_SIZE;
    size_t n_ranges = 0;
    bool vec = tb.vec;
    bool in_place_any = false;
    for (int t = 0; t < n_tensors; ++t) {
        const u64 n = tb.td[t].n;
        if (n == 0) continue;
        bool in_place = false;
        for (int j = 0; j < J; ++j) {
            const size_t i = static_cast<size_t>(j) * n_tensors + t;
            OutDesc& o = out[i];
            o.theta = theta ? theta[i] : nullptr;
            o.theta16 = theta_f16 ? theta_f16[i] : nullptr;
            o.mask = mask ? mask[i] : nullptr;
            if (o.theta == tb.td[t].w) {                    // in place: one density only
                if (J > 1) return CONDENSA_ERR_ARG;
                in_place = true;
            } else {
                ranges[n_ranges++] = byte_range(o.theta, n * 4, true);
            }
            ranges[n_ranges++] = byte_range(o.theta16, n * 2, true);
            ranges[n_ranges++] = byte_range(o.mask, n, true);
            if (o.theta && !aligned16(o.theta)) vec = false;
            if (o.theta16 && (reinterpret_cast<uintptr_t>(o.theta16) & 7u)) vec = false;
            if (o.mask && (reinterpret_cast<uintptr_t>(o.mask) & 3u)) vec = false;
        }
        ranges[n_ranges++] = byte_range(tb.td[t].w, n * 4, in_place);
        in_place_any = in_place_any || in_place;
    }
    ranges[n_ranges++] = byte_range(workspace_dev, workspace_bytes < L.total ? workspace_bytes : L.total, true);
    ranges[n_ranges++] = byte_range(results_dev, static_cast<u64>(L.n_slots) * sizeof(condensa_select), true);
    if (ranges_conflict(ranges, n_ranges)) return CONDENSA_ERR_ARG;
    rc = check_workspace(workspace_dev, workspace_bytes, L);
    if (rc != CONDENSA_OK) return no_alloc ? CONDENSA_ERR_SIZE : rc;

    const bool window = !no_alloc && want_window(tb.N, per_tensor, J, false, cfg);
    Slot* slots = arena.array<Slot>(static_cast<size_t>(L.n_slots) + 3);
    char* up = arena.array<char>(L.upload_bytes);
    if (!slots || !up) return CONDENSA_ERR_SIZE;
    for (int g = 0; g < L.n_groups; ++g)
        for (int j = 0; j < J; ++j) {
            const u64 n = per_tensor ? tb.td[g].n : tb.N;
            init_slot(&slots[static_cast<size_t>(g) * J + j], n, kept_count(densities[j], n), window ? 2u : 1u);
        }
    const size_t n_up_slots = static_cast<size_t>(L.n_slots) + ((window && J == 1) ? 3 : 0);
    if (window && J == 1) init_sample_slots(slots + L.n_slots, slots[0], cfg[CONDENSA_OPT_WINDOW_MARGIN]);

    // one upload: [tensor table | output table | rankings]
    std::memcpy(up + L.td, tb.td, static_cast<size_t>(tb.n_td) * sizeof(TensorDesc));
    std::memcpy(up + L.out, out, n_out * sizeof(OutDesc));
    std::memcpy(up + L.slots, slots, n_up_slots * sizeof(Slot));
    hipStream_t st = static_cast<hipStream_t>(stream);
    rc = no_alloc ? poke_upload(workspace_dev, up, L.upload_bytes, st) : stage_upload(workspace_dev, up, L.upload_bytes, st);
    if (rc != CONDENSA_OK) return rc;
    hipLaunchKernelGGL(k_prepare, dim3(fill_grid(L.zero_bytes / 8)), dim3(kBlock), 0, st,
                       at<u64>(workspace_dev, L.zero_begin), static_cast<u64>(L.zero_bytes / 8),
                       at<TensorDesc>(workspace_dev, L.td), n_tensors, at<u32>(workspace_dev, L.chunk_map), tb.n_chunks);
    CONDENSA_LAUNCH_CHECK();

    DataArgs a{};
    a.td = at<TensorDesc>(workspace_dev, L.td);
    a.slots = at<Slot>(workspace_dev, L.slots);
    a.hist0 = at<u64>(workspace_dev, L.hist0);
    a.histx = at<u64>(workspace_dev, L.histx);
    a.coarse = at<u64>(workspace_dev, L.histc);
    a.tiecnt = at<u32>(workspace_dev, L.tiecnt);
    a.tiehit = at<u32>(workspace_dev, L.tiehit);
    if (L.tl_key) {
        a.tl_cnt = at<u64>(workspace_dev, L.tl_cnt);
        a.tl_key = at<u32>(workspace_dev, L.tl_key);
        a.tl_idx = at<u64>(workspace_dev, L.tl_idx);
        a.small_cap = L.small_cap;
    }
    a.ctl = at<Control>(workspace_dev, L.ctl);
    a.chunk_map = at<u32>(workspace_dev, L.chunk_map);
    a.n_chunks = tb.n_chunks;
    a.N = tb.N;
    a.n_tensors = n_tensors;
    a.J = J;
    a.per_tensor = per_tensor ? 1 : 0;
    a.only_failed = 0;
    a.streaming = (tb.N * 4u >= (static_cast<u64>(512) << 20)) ? 1 : 0;            // well beyond the 256 MB last-level cache
    a.mu = 0.0f;
    a.merged = per_tensor ? 0 : 1;

    // One density on the window path: selection and apply share one sweep unless theta overwrites the weights.
    const bool fuse = window && J == 1 && any_out && tb.n_chunks > 0 && slots[0].k > 0 && !in_place_any &&
                      cfg[CONDENSA_OPT_FUSED_SWEEP] == 0;
    WindowArgs wargs{};
    FusedRequest fr{at<OutDesc>(workspace_dev, L.out), vec, false, &wargs};
    rc = tb.vec ? run_selection<false, true>(a, L, workspace_dev, window, L.n_slots, L.n_groups, results_dev, st, cfg, fuse ? &fr : nullptr)
                : run_selection<false, false>(a, L, workspace_dev, window, L.n_slots, L.n_groups, results_dev, st, cfg, fuse ? &fr : nullptr);
    if (rc != CONDENSA_OK) return rc;

    if (fuse) {
        PhaseTimer timer(CONDENSA_PHASE_APPLY, st, cfg);
        const OutDesc* od = at<OutDesc>(workspace_dev, L.out);
        hipLaunchKernelGGL((k_window_fixup<false, false>), dim3(wargs.n_segs * kFixupParts), dim3(kBlock), 0, st, a, wargs);
        CONDENSA_LAUNCH_CHECK();
        const u64 n_tiles = tb.n_chunks * kSubPerChunk;
        const unsigned grid = static_cast<unsigned>(n_tiles < 4096 ? n_tiles : 4096);
        if (vec) hipLaunchKernelGGL((k_prune_apply_gated<true>), dim3(grid), dim3(kBlock), 0, st, a, od, n_tiles);
        else     hipLaunchKernelGGL((k_prune_apply_gated<false>), dim3(grid), dim3(kBlock), 0, st, a, od, n_tiles);
        CONDENSA_LAUNCH_CHECK();
    } else if (any_out && tb.n_chunks > 0) {
        PhaseTimer timer(CONDENSA_PHASE_APPLY, st, cfg);
        const OutDesc* od = at<OutDesc>(workspace_dev, L.out);
        if (vec) hipLaunchKernelGGL((k_prune_apply<true>), dim3(static_cast<unsigned>(tb.n_chunks * kSubPerChunk)), dim3(kBlock), 0, st, a, od);
        else     hipLaunchKernelGGL((k_prune_apply<false>), dim3(static_cast<unsigned>(tb.n_chunks * kSubPerChunk)), dim3(kBlock), 0, st, a, od);
        CONDENSA_LAUNCH_CHECK();
    }
    return CONDENSA_OK;
}

}  // namespace condensa

using namespace condensa;

// =====================================================================================================

extern "C" {

condensa_status condensa_config_init(condensa_config* config) {
    if (config == nullptr) return CONDENSA_ERR_NULL;
    Config c;
    resolve_config(nullptr, &c);
    config->select_path = static_cast<int32_t>(c[CONDENSA_OPT_SELECT_PATH]);
    config->sample_log2 = static_cast<int32_t>(c[CONDENSA_OPT_SAMPLE_LOG2]);
    config->window_margin = static_cast<int32_t>(c[CONDENSA_OPT_WINDOW_MARGIN]);
    config->cand_shift = static_cast<int32_t>(c[CONDENSA_OPT_CAND_SHIFT]);
    config->profile = static_cast<int32_t>(c[CONDENSA_OPT_PROFILE]);
    config->apply_threads = static_cast<int32_t>(c[CONDENSA_OPT_APPLY_THREADS]);
    config->fused_sweep = static_cast<int32_t>(c[CONDENSA_OPT_FUSED_SWEEP]);
    config->reserved = 0;
    return CONDENSA_OK;
}

size_t condensa_workspace_bytes(int op, uint64_t total_elems, uint64_t n_structures, int n_tensors,
                                int n_densities, int scope, const condensa_config* config) {
    if (op < CONDENSA_OP_PRUNE || op > CONDENSA_OP_LC_SGD_STEP) return 0;
    if (op == CONDENSA_OP_QUANTIZE) return 0;
    if (n_tensors < 0 || n_tensors > CONDENSA_MAX_TENSORS) return 0;
    if (n_densities < 1 || n_densities > CONDENSA_MAX_DENSITIES) return 0;
    if (scope != CONDENSA_SCOPE_GLOBAL && scope != CONDENSA_SCOPE_PER_TENSOR) return 0;
    if (total_elems > kMaxElems || n_structures > total_elems) return 0;
    Config cfg;
    if (resolve_config(config, &cfg) != CONDENSA_OK) return 0;
    return make_layout(op, total_elems, n_structures, n_tensors, n_densities, scope, cfg).total;
}

condensa_status condensa_prune(const condensa_tensor* tensors, int n_tensors, const double* densities,
                               int n_densities, int scope, float* const* theta, uint16_t* const* theta_f16,
                               uint8_t* const* mask, condensa_select* results_dev, void* workspace_dev,
                               size_t workspace_bytes, void* stream, const condensa_config* config) {
    Config cfg;
    const condensa_status rc = resolve_config(config, &cfg);
    if (rc != CONDENSA_OK) return rc;
    HostArena arena;
    return prune_impl(tensors, n_tensors, densities, n_densities, scope, theta, theta_f16, mask, results_dev,
                      workspace_dev, workspace_bytes, stream, cfg, arena, false);
}

condensa_status condensa_prune_static(const condensa_tensor* tensors, int n_tensors, const double* densities,
                                      int n_densities, float* const* theta, uint16_t* const* theta_f16,
                                      uint8_t* const* mask, condensa_select* results_dev, void* stream) {
    if (n_tensors < 0 || n_tensors > CONDENSA_STATIC_MAX_TENSORS) return CONDENSA_ERR_SIZE;
    if (n_densities < 1 || n_densities > CONDENSA_STATIC_MAX_DENSITIES) return CONDENSA_ERR_SIZE;
    if (n_tensors > 0 && tensors == nullptr) return CONDENSA_ERR_NULL;
    u64 total = 0;
    for (int t = 0; t < n_tensors; ++t) {
        u64 n;
        if (!tensor_elems(tensors[t], &n)) return CONDENSA_ERR_SHAPE;
        total += n;
        if (total > CONDENSA_STATIC_MAX_ELEMS) return CONDENSA_ERR_SIZE;
    }
    // built-in settings: nothing of the process-wide defaults applies (no event is created for phase timing)
    Config cfg{};
    cfg.v[CONDENSA_OPT_SELECT_PATH] = 1;
    cfg.v[CONDENSA_OPT_WINDOW_MARGIN] = 80;
    void* ws = nullptr;
    const condensa_status rc = scratch_for_current_device(&ws);
    if (rc != CONDENSA_OK) return rc;
    // host tables on this stack frame: tensor table, output table, rankings, their upload image, byte ranges
    constexpr size_t kHostBytes =
        static_cast<size_t>(CONDENSA_STATIC_MAX_TENSORS + 1) * sizeof(TensorDesc) * 2 +
        static_cast<size_t>(CONDENSA_STATIC_MAX_TENSORS) * CONDENSA_STATIC_MAX_DENSITIES * sizeof(OutDesc) * 2 +
        static_cast<size_t>(CONDENSA_STATIC_MAX_DENSITIES + 2 * kMaxJ) * sizeof(Slot) * 2 +
        (static_cast<size_t>(CONDENSA_STATIC_MAX_TENSORS) * (1 + 3 * CONDENSA_STATIC_MAX_DENSITIES) + 2) * sizeof(ByteRange) +
        4096;
    alignas(64) char host[kHostBytes];
    HostArena arena(host, sizeof(host));
    return prune_impl(tensors, n_tensors, densities, n_densities, CONDENSA_SCOPE_GLOBAL, theta, theta_f16, mask,
                      results_dev, ws, kScratchBytes, stream, cfg, arena, true);
}

}  // extern "C" (reopened below)

namespace condensa {

static condensa_status lc_step_impl(bool pq, const condensa_tensor* tensors, int n_tensors, float* const* lambda,
                                    float* const* lambda_out, float mu, double density, float* const* theta,
                                    uint16_t* const* theta_f16, float* const* grad, uint8_t* const* mask,
                                    uint64_t* nnz_dev, condensa_select* result_dev, void* workspace_dev,
                                    size_t workspace_bytes, void* stream, const condensa_config* config) {
    Config cfg;
    condensa_status rc = resolve_config(config, &cfg);
    if (rc != CONDENSA_OK) return rc;
    if (result_dev == nullptr) return CONDENSA_ERR_NULL;
    if (n_tensors > 0 && lambda == nullptr) return CONDENSA_ERR_NULL;
    if (!density_ok(density)) return CONDENSA_ERR_DENSITY;
    if (!(mu > 0.0f) || !std::isfinite(mu)) return CONDENSA_ERR_DENSITY;
    HostArena arena;
    Tables tb;
    rc = build_tensor_table(tensors, n_tensors, &tb, arena);
    if (rc != CONDENSA_OK) return rc;
    const Layout L = make_layout(CONDENSA_OP_LC_STEP, tb.N, 0, n_tensors, 1, CONDENSA_SCOPE_GLOBAL, cfg);

    std::vector<OutDesc> out(static_cast<size_t>(n_tensors > 0 ? n_tensors : 1), OutDesc{});
    std::vector<ByteRange> ranges;
    ranges.reserve(static_cast<size_t>(n_tensors) * 7 + 2);
    bool vec = tb.vec;
    bool in_place_any = false;
    for (int t = 0; t < n_tensors; ++t) {
        TensorDesc& d = tb.td[t];
        if (d.n == 0) continue;
        if (lambda[t] == nullptr) return CONDENSA_ERR_NULL;
        d.lam = lambda[t];
        d.lam_out = lambda_out ? lambda_out[t] : lambda[t];
        if (d.lam_out == nullptr) return CONDENSA_ERR_NULL;
        d.grad = grad ? grad[t] : nullptr;
        OutDesc& o = out[t];
        o.theta = theta ? theta[t] : nullptr;
        o.theta16 = (pq && theta_f16) ? theta_f16[t] : nullptr;
        o.mask = mask ? mask[t] : nullptr;
        // theta, grad, mask, theta16 and a separate lambda_out must be disjoint from everything else; lambda
        // updated in place is a written range, so it must not overlap the weights either
        const bool in_place = (d.lam_out == d.lam);
        in_place_any = in_place_any || in_place;
        ranges.push_back(byte_range(d.w, d.n * 4, false));
        ranges.push_back(byte_range(d.lam, d.n * 4, in_place));
        if (!in_place) ranges.push_back(byte_range(d.lam_out, d.n * 4, true));
        ranges.push_back(byte_range(o.theta, d.n * 4, true));
        ranges.push_back(byte_range(d.grad, d.n * 4, true));
        ranges.push_back(byte_range(o.mask, d.n, true));
        ranges.push_back(byte_range(o.theta16, d.n * 2, true));
        if (!aligned16(d.lam) || !aligned16(d.lam_out)) vec = false;
        if (o.theta && !aligned16(o.theta)) vec = false;
        if (d.grad && !aligned16(d.grad)) vec = false;
        if (o.mask && (reinterpret_cast<uintptr_t>(o.mask) & 3u)) vec = false;
        if (o.theta16 && (reinterpret_cast<uintptr_t>(o.theta16) & 7u)) vec = false;
    }
    ranges.push_back(byte_range(workspace_dev, workspace_bytes < L.total ? workspace_bytes : L.total, true));
    ranges.push_back(byte_range(result_dev, sizeof(condensa_select), true));
    ranges.push_back(byte_range(nnz_dev, sizeof(uint64_t), true));
    if (ranges_conflict(ranges.data(), ranges.size())) return CONDENSA_ERR_ARG;
    rc = check_workspace(workspace_dev, workspace_bytes, L);
    if (rc != CONDENSA_OK) return rc;
    const bool window = want_window(tb.N, false, 1, true, cfg);
    Slot slot4[4];
    Slot& slot = slot4[0];
    init_slot(&slot, tb.N, kept_count(density, tb.N), window ? 2u : 1u);
    if (window) init_sample_slots(slot4 + 1, slot, cfg[CONDENSA_OPT_WINDOW_MARGIN]);

    std::vector<char> up(L.upload_bytes, 0);
    std::memcpy(up.data() + L.td, tb.td, static_cast<size_t>(tb.n_td) * sizeof(TensorDesc));
    std::memcpy(up.data() + L.out, out.data(), out.size() * sizeof(OutDesc));
    std::memcpy(up.data() + L.slots, slot4, (window ? 4 : 1) * sizeof(Slot));
    hipStream_t st = static_cast<hipStream_t>(stream);
    rc = stage_upload(workspace_dev, up.data(), L.upload_bytes, st);
    if (rc != CONDENSA_OK) return rc;
    hipLaunchKernelGGL(k_prepare, dim3(fill_grid(L.zero_bytes / 8)), dim3(kBlock), 0, st,
                       at<u64>(workspace_dev, L.zero_begin), static_cast<u64>(L.zero_bytes / 8),
                       at<TensorDesc>(workspace_dev, L.td), n_tensors, at<u32>(workspace_dev, L.chunk_map), tb.n_chunks);
    CONDENSA_LAUNCH_CHECK();

    DataArgs a{};
    a.td = at<TensorDesc>(workspace_dev, L.td);
    a.slots = at<Slot>(workspace_dev, L.slots);
    a.hist0 = at<u64>(workspace_dev, L.hist0);
    a.histx = at<u64>(workspace_dev, L.histx);
    a.coarse = at<u64>(workspace_dev, L.histc);
    a.tiecnt = at<u32>(workspace_dev, L.tiecnt);
    a.tiehit = at<u32>(workspace_dev, L.tiehit);
    if (L.tl_key) {
        a.tl_cnt = at<u64>(workspace_dev, L.tl_cnt);
        a.tl_key = at<u32>(workspace_dev, L.tl_key);
        a.tl_idx = at<u64>(workspace_dev, L.tl_idx);
        a.small_cap = L.small_cap;
    }
    a.ctl = at<Control>(workspace_dev, L.ctl);
    a.chunk_map = at<u32>(workspace_dev, L.chunk_map);
    a.n_chunks = tb.n_chunks;
    a.N = tb.N;
    a.n_tensors = n_tensors;
    a.J = 1;
    a.per_tensor = 0;
    a.only_failed = 0;
    a.streaming = (tb.N * 8u >= (static_cast<u64>(512) << 20)) ? 1 : 0;            // w and lambda: well beyond the 256 MB last-level cache
    a.mu = mu;
    a.merged = 1;
    // counters of the apply sweeps' non-zero codes: the last row of the segment counters (rows 1.. belong to the
    // sweeps of several densities, which the L-C step never runs)
    a.nnz_seg = (pq && nnz_dev) ? at<u64>(workspace_dev, L.seg) + static_cast<size_t>(kSegs) * (1 + kMaxJ) : nullptr;

    // the selection sweeps read w and lambda only, so their vector path depends on those alone
    bool vec_in = tb.vec;
    for (int t = 0; t < n_tensors; ++t)
        if (tb.td[t].n > 0 && !aligned16(tb.td[t].lam)) vec_in = false;
    // Window path: selection and apply share one sweep unless lambda is updated in place (a failed window
    // needs the inputs again).
    const bool fuse = window && tb.n_chunks > 0 && slot.k > 0 && !in_place_any && cfg[CONDENSA_OPT_FUSED_SWEEP] == 0;
    WindowArgs wargs{};
    FusedRequest fr{at<OutDesc>(workspace_dev, L.out), vec, pq, &wargs};
    rc = vec_in ? run_selection<true, true>(a, L, workspace_dev, window, 1, 1, result_dev, st, cfg, fuse ? &fr : nullptr)
                : run_selection<true, false>(a, L, workspace_dev, window, 1, 1, result_dev, st, cfg, fuse ? &fr : nullptr);
    if (rc != CONDENSA_OK) return rc;

    if (fuse) {
        PhaseTimer timer(CONDENSA_PHASE_APPLY, st, cfg);
        const OutDesc* od = at<OutDesc>(workspace_dev, L.out);
        if (pq) hipLaunchKernelGGL((k_window_fixup<true, true>), dim3(wargs.n_segs * kFixupParts), dim3(kBlock), 0, st, a, wargs);
        else    hipLaunchKernelGGL((k_window_fixup<true, false>), dim3(wargs.n_segs * kFixupParts), dim3(kBlock), 0, st, a, wargs);
        CONDENSA_LAUNCH_CHECK();
        const u64 n_tiles = tb.n_chunks * (kChunk / 256);
        const dim3 grid(static_cast<unsigned>(n_tiles < 16384 ? n_tiles : 16384));
        if (pq && vec)  hipLaunchKernelGGL((k_lc_apply_gated<true, true>), grid, dim3(64), 0, st, a, od, n_tiles);
        else if (pq)    hipLaunchKernelGGL((k_lc_apply_gated<false, true>), grid, dim3(64), 0, st, a, od, n_tiles);
        else if (vec)   hipLaunchKernelGGL((k_lc_apply_gated<true, false>), grid, dim3(64), 0, st, a, od, n_tiles);
        else            hipLaunchKernelGGL((k_lc_apply_gated<false, false>), grid, dim3(64), 0, st, a, od, n_tiles);
        CONDENSA_LAUNCH_CHECK();
    } else if (tb.n_chunks > 0) {
        PhaseTimer timer(CONDENSA_PHASE_APPLY, st, cfg);
        const OutDesc* od = at<OutDesc>(workspace_dev, L.out);
        const int64_t at_opt = cfg[CONDENSA_OPT_APPLY_THREADS];
        const unsigned nc = static_cast<unsigned>(tb.n_chunks);
        // measured on the 1.2 G-weight workload: 64 threads 3.94 ms, 256 threads 4.28 ms, 128 threads 4.55 ms
        if (pq) {
            if (vec) hipLaunchKernelGGL((k_lc_apply<true, 64, true>), dim3(nc * (kChunk / 256)), dim3(64), 0, st, a, od);
            else     hipLaunchKernelGGL((k_lc_apply<false, 256, true>), dim3(nc * (kChunk / 1024)), dim3(256), 0, st, a, od);
        }
        else if (vec && at_opt == 256) hipLaunchKernelGGL((k_lc_apply<true, 256, false>), dim3(nc * (kChunk / 1024)), dim3(256), 0, st, a, od);
        else if (vec && at_opt == 128) hipLaunchKernelGGL((k_lc_apply<true, 128, false>), dim3(nc * (kChunk / 512)), dim3(128), 0, st, a, od);
        else if (vec)                  hipLaunchKernelGGL((k_lc_apply<true, 64, false>), dim3(nc * (kChunk / 256)), dim3(64), 0, st, a, od);
        else                           hipLaunchKernelGGL((k_lc_apply<false, 256, false>), dim3(nc * (kChunk / 1024)), dim3(256), 0, st, a, od);
        CONDENSA_LAUNCH_CHECK();
    }
    if (pq && nnz_dev) {
        hipLaunchKernelGGL(k_nnz_finish, dim3(1), dim3(kBlock), 0, st, a, at<u64>(workspace_dev, L.seg) + kSegs,
                           (fuse && tb.n_chunks > 0) ? 1 : 0, nnz_dev);
        CONDENSA_LAUNCH_CHECK();
    }
    return CONDENSA_OK;
}

}  // namespace condensa

extern "C" {

condensa_status condensa_lc_step(const condensa_tensor* tensors, int n_tensors, float* const* lambda,
                                 float* const* lambda_out, float mu, double density, float* const* theta,
                                 float* const* grad, uint8_t* const* mask, condensa_select* result_dev,
                                 void* workspace_dev, size_t workspace_bytes, void* stream,
                                 const condensa_config* config) {
    return lc_step_impl(false, tensors, n_tensors, lambda, lambda_out, mu, density, theta, nullptr, grad, mask,
                        nullptr, result_dev, workspace_dev, workspace_bytes, stream, config);
}

condensa_status condensa_lc_step_pq(const condensa_tensor* tensors, int n_tensors, float* const* lambda,
                                    float* const* lambda_out, float mu, double density, float* const* theta,
                                    uint16_t* const* theta_f16, float* const* grad, uint8_t* const* mask,
                                    uint64_t* nnz_dev, condensa_select* result_dev, void* workspace_dev,
                                    size_t workspace_bytes, void* stream, const condensa_config* config) {
    return lc_step_impl(true, tensors, n_tensors, lambda, lambda_out, mu, density, theta, theta_f16, grad, mask,
                        nnz_dev, result_dev, workspace_dev, workspace_bytes, stream, config);
}

condensa_status condensa_count_nonzero(const condensa_tensor* tensors, int n_tensors, int kind,
                                       uint64_t* count_dev, void* workspace_dev, size_t workspace_bytes,
                                       void* stream, const condensa_config* config) {
    Config cfg;
    condensa_status rc = resolve_config(config, &cfg);
    if (rc != CONDENSA_OK) return rc;
    if (count_dev == nullptr) return CONDENSA_ERR_NULL;
    if (kind < CONDENSA_COUNT_F32 || kind > CONDENSA_COUNT_CODES8) return CONDENSA_ERR_ARG;
    HostArena arena;
    Tables tb;
    rc = build_tensor_table(tensors, n_tensors, &tb, arena);
    if (rc != CONDENSA_OK) return rc;
    const Layout L = make_layout(CONDENSA_OP_COUNT_NONZERO, tb.N, 0, n_tensors, 1, CONDENSA_SCOPE_GLOBAL, cfg);
    rc = check_workspace(workspace_dev, workspace_bytes, L);
    if (rc != CONDENSA_OK) return rc;
    bool vec = true;
    std::vector<ByteRange> ranges;
    const u64 elem_bytes = kind == CONDENSA_COUNT_F32 ? 4 : (kind == CONDENSA_COUNT_CODES16 ? 2 : 1);
    for (int t = 0; t < n_tensors; ++t) {
        if (tb.td[t].n > 0 && (reinterpret_cast<uintptr_t>(tb.td[t].w) & 15u)) vec = false;
        ranges.push_back(byte_range(tb.td[t].w, tb.td[t].n * elem_bytes, false));
    }
    ranges.push_back(byte_range(workspace_dev, workspace_bytes < L.total ? workspace_bytes : L.total, true));
    ranges.push_back(byte_range(count_dev, sizeof(uint64_t), true));
    if (ranges_conflict(ranges.data(), ranges.size())) return CONDENSA_ERR_ARG;
    std::vector<char> up(L.upload_bytes, 0);
    std::memcpy(up.data() + L.td, tb.td, static_cast<size_t>(tb.n_td) * sizeof(TensorDesc));
    hipStream_t st = static_cast<hipStream_t>(stream);
    rc = stage_upload(workspace_dev, up.data(), L.upload_bytes, st);
    if (rc != CONDENSA_OK) return rc;
    hipLaunchKernelGGL(k_prepare, dim3(fill_grid(L.zero_bytes / 8)), dim3(kBlock), 0, st,
                       at<u64>(workspace_dev, L.zero_begin), static_cast<u64>(L.zero_bytes / 8),
                       at<TensorDesc>(workspace_dev, L.td), n_tensors, at<u32>(workspace_dev, L.chunk_map), tb.n_chunks);
    CONDENSA_LAUNCH_CHECK();
    DataArgs a{};
    a.td = at<TensorDesc>(workspace_dev, L.td);
    a.chunk_map = at<u32>(workspace_dev, L.chunk_map);
    a.n_chunks = tb.n_chunks;
    a.N = tb.N;
    a.n_tensors = n_tensors;
    u64* partial = at<u64>(workspace_dev, L.hist0);            // kBins words, cleared by k_prepare
    const unsigned blocks = static_cast<unsigned>(tb.n_chunks < static_cast<u64>(kBins) ? (tb.n_chunks ? tb.n_chunks : 1) : kBins);
    if (tb.n_chunks > 0) {
        if (kind == CONDENSA_COUNT_CODES8) {
            if (vec) hipLaunchKernelGGL((k_count_nonzero<2, true>), dim3(blocks), dim3(kBlock), 0, st, a, partial);
            else     hipLaunchKernelGGL((k_count_nonzero<2, false>), dim3(blocks), dim3(kBlock), 0, st, a, partial);
        } else if (kind == CONDENSA_COUNT_CODES16) {
            if (vec) hipLaunchKernelGGL((k_count_nonzero<1, true>), dim3(blocks), dim3(kBlock), 0, st, a, partial);
            else     hipLaunchKernelGGL((k_count_nonzero<1, false>), dim3(blocks), dim3(kBlock), 0, st, a, partial);
        } else {
            if (vec) hipLaunchKernelGGL((k_count_nonzero<0, true>), dim3(blocks), dim3(kBlock), 0, st, a, partial);
            else     hipLaunchKernelGGL((k_count_nonzero<0, false>), dim3(blocks), dim3(kBlock), 0, st, a, partial);
        }
        CONDENSA_LAUNCH_CHECK();
    }
    hipLaunchKernelGGL(k_sum_partials, dim3(1), dim3(kBlock), 0, st, partial, blocks, count_dev);
    CONDENSA_LAUNCH_CHECK();
    return CONDENSA_OK;
}

}  // extern "C" (reopened below)

// ---- structure pruning (filters, 2-D blocks) ---------------------------------------------------------

namespace condensa {

static condensa_status run_structure_prune(int op, Tables& tb, int n_tensors, double density, int scope,
                                           float* const* theta, uint8_t* const* mask, double* sumsq_dev,
                                           float* norms_dev, int32_t* keep_idx_dev, uint8_t* structure_mask_dev,
                                           condensa_select* results_dev, void* workspace_dev,
                                           size_t workspace_bytes, void* stream, const Config& cfg) {
    const bool per_tensor = (scope == CONDENSA_SCOPE_PER_TENSOR);
    if (per_tensor && n_tensors == 0) return CONDENSA_OK;
    const Layout L = make_layout(op, tb.N, tb.F, n_tensors, 1, scope, cfg);

    std::vector<OutDesc> out(static_cast<size_t>(n_tensors > 0 ? n_tensors : 1), OutDesc{});
    std::vector<ByteRange> ranges;
    ranges.reserve(static_cast<size_t>(n_tensors) * 3 + 6);
    bool vec = tb.vec;
    for (int t = 0; t < n_tensors; ++t) {
        const u64 n = tb.td[t].n;
        if (n == 0) continue;
        OutDesc& o = out[t];
        o.theta = theta ? theta[t] : nullptr;
        o.mask = mask ? mask[t] : nullptr;
        const bool in_place = (o.theta == tb.td[t].w);       // the aggregates are complete before the apply sweep
        if (!in_place) ranges.push_back(byte_range(o.theta, n * 4, true));
        ranges.push_back(byte_range(o.mask, n, true));
        ranges.push_back(byte_range(tb.td[t].w, n * 4, in_place));
        if (o.theta && !aligned16(o.theta)) vec = false;
        if (o.mask && (reinterpret_cast<uintptr_t>(o.mask) & 3u)) vec = false;
    }
    ranges.push_back(byte_range(sumsq_dev, tb.F * 8, true));
    ranges.push_back(byte_range(norms_dev, tb.F * 4, true));
    ranges.push_back(byte_range(keep_idx_dev, tb.F * 4, true));
    ranges.push_back(byte_range(structure_mask_dev, tb.F, true));
    ranges.push_back(byte_range(workspace_dev, workspace_bytes < L.total ? workspace_bytes : L.total, true));
    ranges.push_back(byte_range(results_dev, static_cast<u64>(L.n_slots) * sizeof(condensa_select), true));
    if (ranges_conflict(ranges.data(), ranges.size())) return CONDENSA_ERR_ARG;
    condensa_status rc = check_workspace(workspace_dev, workspace_bytes, L);
    if (rc != CONDENSA_OK) return rc;
    std::vector<Slot> slots(static_cast<size_t>(L.n_slots) + 3);
    for (int g = 0; g < L.n_groups; ++g) {
        const u64 n = per_tensor ? tb.td[g].n_struct : tb.F;
        init_slot(&slots[g], n, kept_count(density, n), 1u);
    }
    // One sweep for aggregation AND apply (k_struct_fused.h): 8x8 blocks, every matrix a whole number of 64-block
    // runs wide, 128-bit accesses everywhere, outputs apart from the weights, a threshold strictly inside the
    // population, and enough blocks for the sample to pay (or the form asked for).
    bool fused = !per_tensor && (theta || mask) && vec && tb.F > kSmallGroup && slots[0].k > 0 && slots[0].k < tb.F &&
                 (cfg[CONDENSA_OPT_SELECT_PATH] == 2 || (cfg[CONDENSA_OPT_SELECT_PATH] == 0 && tb.F >= (static_cast<u64>(1) << 20))) &&
                 cfg[CONDENSA_OPT_FUSED_SWEEP] == 0;
    for (int t = 0; t < n_tensors && fused; ++t) {
        const TensorDesc& d = tb.td[t];
        if (d.n == 0) continue;
        const bool ok = d.d[0] == 1 && d.d[1] == 1 && d.b[2] == 8 && d.b[3] == 8 && d.d[2] % 8 == 0 && d.d[3] % 512 == 0 &&
                        aligned16(d.w) && d.n <= 0xFFFFFFFFull && out[t].theta != d.w;
        if (!ok) fused = false;
    }
    if (fused) {
        init_sample_slots(&slots[L.n_slots], slots[0], cfg[CONDENSA_OPT_WINDOW_MARGIN]);
        slots[0].path = 2;
    }
    std::vector<char> up(L.upload_bytes, 0);
    std::memcpy(up.data() + L.td, tb.td, static_cast<size_t>(tb.n_td) * sizeof(TensorDesc));
    std::memcpy(up.data() + L.out, out.data(), out.size() * sizeof(OutDesc));
    std::memcpy(up.data() + L.slots, slots.data(), (static_cast<size_t>(L.n_slots) + (fused ? 3 : 0)) * sizeof(Slot));
    hipStream_t st = static_cast<hipStream_t>(stream);
    rc = stage_upload(workspace_dev, up.data(), L.upload_bytes, st);
    if (rc != CONDENSA_OK) return rc;
    hipLaunchKernelGGL(k_prepare, dim3(fill_grid(L.zero_bytes / 8)), dim3(kBlock), 0, st,
                       at<u64>(workspace_dev, L.zero_begin), static_cast<u64>(L.zero_bytes / 8),
                       at<TensorDesc>(workspace_dev, L.td), n_tensors, at<u32>(workspace_dev, L.chunk_map), tb.n_chunks);
    CONDENSA_LAUNCH_CHECK();

    StructArgs a{};
    a.td = at<TensorDesc>(workspace_dev, L.td);
    a.slots = at<Slot>(workspace_dev, L.slots);
    a.histx = at<u64>(workspace_dev, L.histx);
    a.tiecnt = at<u32>(workspace_dev, L.tiecnt);
    a.ctl = at<Control>(workspace_dev, L.ctl);
    a.keys = at<u64>(workspace_dev, L.skeys);
    a.smask = at<u8>(workspace_dev, L.smask);
    a.sblock = at<u32>(workspace_dev, L.sblock);
    a.chunk_map = at<u32>(workspace_dev, L.chunk_map);
    a.F = tb.F;
    a.n_schunks = tb.n_schunks;
    a.n_chunks = tb.n_chunks;
    a.n_tensors = n_tensors;
    a.per_tensor = per_tensor ? 1 : 0;
    a.merged = per_tensor ? 0 : 1;
    a.hist_base = at<u64>(workspace_dev, L.hist0);
    a.coarse = at<u64>(workspace_dev, L.histc);

    const unsigned sblocks = static_cast<unsigned>((tb.F + kBlock - 1) / kBlock);
    const unsigned mtiles = static_cast<unsigned>((tb.F + kMaskTile - 1) / kMaskTile);
    // groups of at most kSmallGroup structures: one workgroup per group ranks, masks and lists them
    bool small = tb.F > 0 && cfg[CONDENSA_OPT_SELECT_PATH] != 1;
    if (per_tensor) { for (int t = 0; t < n_tensors && small; ++t) if (tb.td[t].n_struct > kSmallGroup) small = false; }
    else if (tb.F > kSmallGroup) small = false;
    bool finished = false;                                  // the ranking's record is written (k_struct_list_finish)
    StructWindowArgs sw{};
    if (fused) {
        sw.sample = at<u32>(workspace_dev, L.sample);
        sw.n_units = (L.sample_cap < tb.F ? L.sample_cap : tb.F) & ~static_cast<u64>(3);   // whole units of four blocks
        sw.stride = tb.F / sw.n_units;
        sw.wslots = a.slots + L.n_slots;
        sw.seg_cnt = at<u64>(workspace_dev, L.seg);
        sw.seg_above = sw.seg_cnt + kSegs;
        sw.cand_id = at<u32>(workspace_dev, L.cand_key);
        sw.cand_key = at<u64>(workspace_dev, L.cand_idx);
        sw.n_segs = sblocks < static_cast<unsigned>(kSegs) ? sblocks : static_cast<unsigned>(kSegs);   // at most the sweep's grid
        sw.seg_cap = L.cand_cap / sw.n_segs;
        sw.out = at<OutDesc>(workspace_dev, L.out);
        PhaseTimer timer(CONDENSA_PHASE_SAMPLE, st, cfg);
        ArrayArgs ar{};
        ar.keys = sw.sample; ar.n_host = sw.n_units; ar.slots = sw.wslots; ar.n_slots = 3;
        ar.hist = a.histx + static_cast<u64>(kStructLevels) * kBins;          // [2][3], behind the aggregate ranking's histograms
        ar.shared0 = ar.hist + static_cast<u64>(6) * kBins;
        ar.key_bits = 31; ar.merged = 1;
        ar.hist_base = at<u64>(workspace_dev, L.hist0); ar.coarse = at<u64>(workspace_dev, L.histc);
        u64 sg = (sw.n_units + kSampleHistThreads - 1) / kSampleHistThreads;
        if (sg > 512) sg = 512;
        hipLaunchKernelGGL(k_struct_sample_hist, dim3(static_cast<unsigned>(sg)), dim3(kSampleHistThreads), 0, st, a, sw, ar);
        CONDENSA_LAUNCH_CHECK();
        hipLaunchKernelGGL((k_hist_array<false>), dim3(hist_array_grid(ar.n_host)), dim3(kArrayThreads), 0, st, ar, 1);
        CONDENSA_LAUNCH_CHECK();
        hipLaunchKernelGGL(k_window_bounds, dim3(1), dim3(kBlock), 0, st, ar);
        CONDENSA_LAUNCH_CHECK();
    }
    if (tb.F > 0) {
        {
            PhaseTimer timer(CONDENSA_PHASE_AGGREGATE, st, cfg);
            // every structure one contiguous row (filters, neurons) of some length: staged, coalesced reads
            constexpr u64 kFewRowsMax = 32768;           // up to 1024 workgroups of kFewRows rows
            bool rows = tb.N / tb.F >= 16;
            for (int t = 0; t < n_tensors && rows; ++t) {
                const TensorDesc& d = tb.td[t];
                if (d.n > 0 && !(d.d[1] == 1 && d.d[2] == 1 && d.b[0] == 1 && d.b[3] == d.d[3])) rows = false;
            }
            // every tensor a matrix tiled exactly by 2-D blocks of one width of 4, 8, 16 or 32, rows 16-byte aligned
            u32 tile_w = 0;
            bool tiles = !rows;
            for (int t = 0; t < n_tensors && tiles; ++t) {
                const TensorDesc& d = tb.td[t];
                if (d.n == 0) continue;
                const bool ok = d.d[0] == 1 && d.d[1] == 1 && d.d[2] % d.b[2] == 0 && d.d[3] % d.b[3] == 0 &&
                                (d.b[3] == 4 || d.b[3] == 8 || d.b[3] == 16 || d.b[3] == 32) && (tile_w == 0 || tile_w == d.b[3]) &&
                                aligned16(d.w) && d.d[3] % 4 == 0 && d.n <= 0xFFFFFFFFull;
                if (!ok) tiles = false;
                tile_w = d.b[3];
            }
            if (fused && cfg[CONDENSA_OPT_APPLY_THREADS] == 256)
                hipLaunchKernelGGL((k_struct_tiles_fused<256>), dim3(sblocks), dim3(256), 0, st, a, sw, sumsq_dev, norms_dev);
            else if (fused && cfg[CONDENSA_OPT_APPLY_THREADS] == 128)
                hipLaunchKernelGGL((k_struct_tiles_fused<128>), dim3(static_cast<unsigned>((tb.F + 127) / 128)), dim3(128), 0, st, a, sw, sumsq_dev, norms_dev);
            else if (fused)
                hipLaunchKernelGGL((k_struct_tiles_fused<64>), dim3(static_cast<unsigned>((tb.F + 63) / 64)), dim3(64), 0, st, a, sw, sumsq_dev, norms_dev);
            else if (rows && tb.F <= kFewRowsMax)
                hipLaunchKernelGGL(k_struct_sumsq_rows_few, dim3(static_cast<unsigned>((tb.F + kFewRows - 1) / kFewRows)), dim3(kBlock), 0, st, a, sumsq_dev, norms_dev);
            else if (rows) hipLaunchKernelGGL(k_struct_sumsq_rows, dim3(sblocks), dim3(kBlock), 0, st, a, sumsq_dev, norms_dev);
            else if (tiles && tile_w == 4)  hipLaunchKernelGGL((k_struct_sumsq_tiles<1>), dim3(sblocks), dim3(kBlock), 0, st, a, sumsq_dev, norms_dev);
            else if (tiles && tile_w == 8)  hipLaunchKernelGGL((k_struct_sumsq_tiles<2>), dim3(sblocks), dim3(kBlock), 0, st, a, sumsq_dev, norms_dev);
            else if (tiles && tile_w == 16) hipLaunchKernelGGL((k_struct_sumsq_tiles<4>), dim3(sblocks), dim3(kBlock), 0, st, a, sumsq_dev, norms_dev);
            else if (tiles && tile_w == 32) hipLaunchKernelGGL((k_struct_sumsq_tiles<8>), dim3(sblocks), dim3(kBlock), 0, st, a, sumsq_dev, norms_dev);
            else      hipLaunchKernelGGL(k_struct_sumsq, dim3(sblocks), dim3(kBlock), 0, st, a, sumsq_dev, norms_dev);
            CONDENSA_LAUNCH_CHECK();
        }
        PhaseTimer timer(CONDENSA_PHASE_RESOLVE, st, cfg);
        if (small) {
            hipLaunchKernelGGL(k_struct_small, dim3(L.n_slots), dim3(kSmallThreads), 0, st, a, structure_mask_dev,
                               keep_idx_dev, results_dev);
            CONDENSA_LAUNCH_CHECK();
        }
        if (fused) {
            // rank k - (blocks above the window) among the listed blocks; the levels over all aggregates below are
            // then the fallback and return at once
            hipLaunchKernelGGL(k_struct_window_check, dim3(1), dim3(kBlock), 0, st, a, sw);
            CONDENSA_LAUNCH_CHECK();
            const unsigned lg = sw.n_segs < 256 ? sw.n_segs : 256;
            for (int level = 0; level < n_levels(63); ++level) {
                hipLaunchKernelGGL(k_hist_listed_keys, dim3(lg), dim3(kArrayThreads), 0, st, a, sw, level);
                CONDENSA_LAUNCH_CHECK();
            }
            a.only_failed = 1;
        }
        // moderate rankings on the automatic path: two levels over all aggregates, then a list (k_struct_list.h)
        const bool listed = !per_tensor && !small && !fused && tb.F <= kSmallCallElems && cfg[CONDENSA_OPT_SELECT_PATH] == 0;
        u64 blocks = tb.n_schunks < 1024 ? tb.n_schunks : 1024;
        const u64 cpb = (tb.n_schunks + blocks - 1) / blocks;
        blocks = (tb.n_schunks + cpb - 1) / cpb;
        for (int level = 0; level < (listed ? kStructListLevels : n_levels(63)) && !small; ++level) {
            hipLaunchKernelGGL(k_hist_keys, dim3(static_cast<unsigned>(blocks)), dim3(kBlock), 0, st, a, level, cpb);
            CONDENSA_LAUNCH_CHECK();
            if (a.merged) continue;                            // the next kernel folds this level in itself
            hipLaunchKernelGGL(k_scan_level, dim3(L.n_slots), dim3(kBlock), 0, st, a.slots,
                               static_cast<const u64*>(nullptr), a.histx, 1, 63, level, a.ctl, 0, &a.ctl->need_tie);
            CONDENSA_LAUNCH_CHECK();
        }
        if (listed) {
            StructListArgs l{};
            l.count = at<u64>(workspace_dev, L.seg);
            l.key = at<u64>(workspace_dev, L.cand_idx);
            l.id = at<u32>(workspace_dev, L.cand_key);
            l.cap = L.cand_cap;
            hipLaunchKernelGGL(k_struct_list_collect, dim3(static_cast<unsigned>(tb.n_schunks < 1024 ? tb.n_schunks : 1024)), dim3(kBlock), 0, st, a, l);
            CONDENSA_LAUNCH_CHECK();
            hipLaunchKernelGGL(k_struct_list_finish, dim3(1), dim3(kSmallFinishThreads), 0, st, a, l, results_dev, bits_for(tb.F - 1));
            CONDENSA_LAUNCH_CHECK();
            finished = true;
        } else if (!small) {
            hipLaunchKernelGGL(k_tie_count_keys, dim3(static_cast<unsigned>(tb.n_schunks)), dim3(kBlock), 0, st, a);
            CONDENSA_LAUNCH_CHECK();
        }
    }
    if (!small && !finished) {
        hipLaunchKernelGGL(k_tie_locate_keys, dim3(L.n_slots), dim3(kBlock), 0, st, a, results_dev);
        CONDENSA_LAUNCH_CHECK();
    }
    if (tb.F > 0) {
        if (fused) {
            // the sweep left the keep flags of the blocks outside the window, the fix-up settles the listed ones
            // (and rewrites their theta and mask); the flags come from the keys only if the window failed
            PhaseTimer timer(CONDENSA_PHASE_APPLY, st, cfg);
            hipLaunchKernelGGL(k_struct_fixup, dim3(sw.n_segs * kFixupParts), dim3(kBlock), 0, st, a, sw);
            CONDENSA_LAUNCH_CHECK();
            hipLaunchKernelGGL(k_struct_mask, dim3(mtiles), dim3(kBlock), 0, st, a, structure_mask_dev, static_cast<int>(kMaskFromFlags));
            CONDENSA_LAUNCH_CHECK();
            hipLaunchKernelGGL(k_struct_mask, dim3(mtiles), dim3(kBlock), 0, st, a, structure_mask_dev, static_cast<int>(kMaskIfFailed));
            CONDENSA_LAUNCH_CHECK();
        } else if (!small) {
            hipLaunchKernelGGL(k_struct_mask, dim3(mtiles), dim3(kBlock), 0, st, a, structure_mask_dev, static_cast<int>(kMaskFromKeys));
            CONDENSA_LAUNCH_CHECK();
        }
        if (keep_idx_dev && !small) {
            hipLaunchKernelGGL(k_struct_scan_blocks, dim3(1), dim3(kScanThreads), 0, st, a.sblock, static_cast<u64>(mtiles));
            CONDENSA_LAUNCH_CHECK();
            hipLaunchKernelGGL(k_struct_keep_idx, dim3(mtiles), dim3(kBlock), 0, st, a, keep_idx_dev);
            CONDENSA_LAUNCH_CHECK();
        }
        if (fused) {
            PhaseTimer timer(CONDENSA_PHASE_APPLY, st, cfg);
            const OutDesc* od = at<OutDesc>(workspace_dev, L.out);
            const u64 n_tiles = tb.n_chunks * kSubPerChunk;
            hipLaunchKernelGGL((k_struct_apply_gated<true>), dim3(static_cast<unsigned>(n_tiles < 4096 ? n_tiles : 4096)), dim3(kBlock), 0, st, a, od, n_tiles);
            CONDENSA_LAUNCH_CHECK();
        } else if ((theta || mask) && tb.n_chunks > 0) {
            PhaseTimer timer(CONDENSA_PHASE_APPLY, st, cfg);
            const OutDesc* od = at<OutDesc>(workspace_dev, L.out);
            if (vec) hipLaunchKernelGGL((k_struct_apply<true>), dim3(static_cast<unsigned>(tb.n_chunks * kSubPerChunk)), dim3(kBlock), 0, st, a, od);
            else     hipLaunchKernelGGL((k_struct_apply<false>), dim3(static_cast<unsigned>(tb.n_chunks * kSubPerChunk)), dim3(kBlock), 0, st, a, od);
            CONDENSA_LAUNCH_CHECK();
        }
    }
    return CONDENSA_OK;
}

enum StructKind { kFilters, kNeurons, kNeuronsAndFilters, kBlocks2D, kBlocksND };

// Fills the structure geometry of the tensor table.  Every tensor is seen as 4-D (leading dims 1)
// with a 4-D block; a filter / neuron is the block [1,1,1,len] of the tensor viewed as [F,1,1,len].
static condensa_status add_structure_geometry(const condensa_tensor* tensors, int n_tensors, StructKind kind,
                                              const int32_t* block, int block_ndim, Tables* tb) {
    u64 F = 0, sc = 0;
    for (int t = 0; t < n_tensors; ++t) {
        TensorDesc& d = tb->td[t];
        const condensa_tensor& T = tensors[t];
        d.struct_start = F;
        d.pad = sc;
        for (int i = 0; i < 4; ++i) { d.d[i] = 1; d.b[i] = 1; }
        u64 f = 0;
        if (kind == kFilters || kind == kNeurons || kind == kNeuronsAndFilters) {
            const bool ok = (kind == kFilters) ? T.ndim == 4 : (kind == kNeurons) ? T.ndim == 2 : (T.ndim == 2 || T.ndim == 4);
            if (!ok) return CONDENSA_ERR_SHAPE;
            if (d.n > 0) {
                f = static_cast<u64>(T.shape[0]);
                const u64 len = d.n / f;
                if (len > 0x7FFFFFFFull || f > 0x7FFFFFFFull) return CONDENSA_ERR_SIZE;
                d.d[0] = static_cast<u32>(f); d.d[3] = static_cast<u32>(len); d.b[3] = static_cast<u32>(len);
            }
        } else {
            if (T.ndim != block_ndim) return CONDENSA_ERR_SHAPE;
            const int pad = 4 - T.ndim;
            f = d.n > 0 ? 1 : 0;
            for (int i = 0; i < T.ndim; ++i) {
                const u64 dim = static_cast<u64>(T.shape[i]), blk = static_cast<u64>(block[i]);
                if (dim > 0x7FFFFFFFull) return CONDENSA_ERR_SIZE;
                if (kind == kBlocks2D && dim % blk != 0) return CONDENSA_ERR_SHAPE;
                if (d.n > 0) {
                    d.d[pad + i] = static_cast<u32>(dim);
                    d.b[pad + i] = static_cast<u32>(blk < dim ? blk : dim);
                    f *= (dim + blk - 1) / blk;
                }
            }
        }
        d.fd[kDivD1] = make_fastdiv(d.d[1]); d.fd[kDivD2] = make_fastdiv(d.d[2]); d.fd[kDivD3] = make_fastdiv(d.d[3]);
        d.fd[kDivB0] = make_fastdiv(d.b[0]); d.fd[kDivB1] = make_fastdiv(d.b[1]);
        d.fd[kDivB2] = make_fastdiv(d.b[2]); d.fd[kDivB3] = make_fastdiv(d.b[3]);
        d.n_struct = f;
        F += f;
        sc += (f + kChunk - 1) / kChunk;
    }
    if (F > 0x7FFFFFFFull) return CONDENSA_ERR_SIZE;         // ids are reported as int32
    tb->td[n_tensors].struct_start = F;
    tb->td[n_tensors].pad = sc;
    tb->F = F;
    tb->n_schunks = sc;
    return CONDENSA_OK;
}

static condensa_status structure_entry(StructKind kind, int op, const condensa_tensor* tensors, int n_tensors,
                                       const int32_t* block, int block_ndim, double density, int scope,
                                       float* const* theta, uint8_t* const* mask, double* sumsq_dev,
                                       float* norms_dev, int32_t* keep_idx_dev, uint8_t* structure_mask_dev,
                                       condensa_select* results_dev, void* workspace_dev, size_t workspace_bytes,
                                       void* stream, const condensa_config* config) {
    Config cfg;
    condensa_status rc = resolve_config(config, &cfg);
    if (rc != CONDENSA_OK) return rc;
    if (results_dev == nullptr) return CONDENSA_ERR_NULL;
    if (scope != CONDENSA_SCOPE_GLOBAL && scope != CONDENSA_SCOPE_PER_TENSOR) return CONDENSA_ERR_ARG;
    if (!density_ok(density)) return CONDENSA_ERR_DENSITY;
    if (kind == kBlocks2D || kind == kBlocksND) {
        if (block == nullptr) return CONDENSA_ERR_NULL;
        if (block_ndim < 1 || block_ndim > 4) return CONDENSA_ERR_SHAPE;
        for (int i = 0; i < block_ndim; ++i)
            if (block[i] < 1) return CONDENSA_ERR_SHAPE;
    }
    HostArena arena;
    Tables tb;
    rc = build_tensor_table(tensors, n_tensors, &tb, arena);
    if (rc != CONDENSA_OK) return rc;
    rc = add_structure_geometry(tensors, n_tensors, kind, block, block_ndim, &tb);
    if (rc != CONDENSA_OK) return rc;
    return run_structure_prune(op, tb, n_tensors, density, scope, theta, mask, sumsq_dev, norms_dev, keep_idx_dev,
                               structure_mask_dev, results_dev, workspace_dev, workspace_bytes, stream, cfg);
}

}  // namespace condensa

extern "C" {

condensa_status condensa_filter_prune(const condensa_tensor* tensors, int n_tensors, double density, int scope,
                                      float* const* theta, uint8_t* const* mask, double* sumsq_dev,
                                      float* norms_dev, int32_t* keep_idx_dev, uint8_t* structure_mask_dev,
                                      condensa_select* results_dev, void* workspace_dev, size_t workspace_bytes,
                                      void* stream,
                                      const condensa_config* config) {
    return structure_entry(kFilters, CONDENSA_OP_FILTER_PRUNE, tensors, n_tensors, nullptr, 0, density, scope, theta,
                           mask, sumsq_dev, norms_dev, keep_idx_dev, structure_mask_dev, results_dev, workspace_dev,
                           workspace_bytes, stream, config);
}

condensa_status condensa_neuron_prune(const condensa_tensor* tensors, int n_tensors, double density, int scope,
                                      float* const* theta, uint8_t* const* mask, double* sumsq_dev,
                                      float* norms_dev, int32_t* keep_idx_dev, uint8_t* structure_mask_dev,
                                      condensa_select* results_dev, void* workspace_dev, size_t workspace_bytes,
                                      void* stream,
                                      const condensa_config* config) {
    return structure_entry(kNeurons, CONDENSA_OP_FILTER_PRUNE, tensors, n_tensors, nullptr, 0, density, scope, theta,
                           mask, sumsq_dev, norms_dev, keep_idx_dev, structure_mask_dev, results_dev, workspace_dev,
                           workspace_bytes, stream, config);
}

condensa_status condensa_structure_prune(const condensa_tensor* tensors, int n_tensors, double density, int scope,
                                         float* const* theta, uint8_t* const* mask, double* sumsq_dev,
                                         float* norms_dev, int32_t* keep_idx_dev, uint8_t* structure_mask_dev,
                                         condensa_select* results_dev, void* workspace_dev, size_t workspace_bytes,
                                         void* stream,
                                      const condensa_config* config) {
    return structure_entry(kNeuronsAndFilters, CONDENSA_OP_FILTER_PRUNE, tensors, n_tensors, nullptr, 0, density, scope,
                           theta, mask, sumsq_dev, norms_dev, keep_idx_dev, structure_mask_dev, results_dev,
                           workspace_dev, workspace_bytes, stream, config);
}

condensa_status condensa_block_prune(const condensa_tensor* tensors, int n_tensors, int block_h, int block_w,
                                     double density, int scope, float* const* theta, uint8_t* const* mask,
                                     double* sumsq_dev, float* norms_dev, int32_t* keep_idx_dev,
                                     uint8_t* structure_mask_dev, condensa_select* results_dev,
                                     void* workspace_dev, size_t workspace_bytes, void* stream,
                                      const condensa_config* config) {
    const int32_t block[2] = {block_h, block_w};
    return structure_entry(kBlocks2D, CONDENSA_OP_BLOCK_PRUNE, tensors, n_tensors, block, 2, density, scope, theta,
                           mask, sumsq_dev, norms_dev, keep_idx_dev, structure_mask_dev, results_dev, workspace_dev,
                           workspace_bytes, stream, config);
}

condensa_status condensa_block_prune_nd(const condensa_tensor* tensors, int n_tensors, const int32_t* block_shape,
                                        int block_ndim, double density, int scope, float* const* theta,
                                        uint8_t* const* mask, double* sumsq_dev, float* norms_dev,
                                        int32_t* keep_idx_dev, uint8_t* structure_mask_dev,
                                        condensa_select* results_dev, void* workspace_dev, size_t workspace_bytes,
                                        void* stream,
                                      const condensa_config* config) {
    return structure_entry(kBlocksND, CONDENSA_OP_BLOCK_PRUNE, tensors, n_tensors, block_shape, block_ndim, density,
                           scope, theta, mask, sumsq_dev, norms_dev, keep_idx_dev, structure_mask_dev, results_dev,
                           workspace_dev, workspace_bytes, stream, config);
}

}  // extern "C"

namespace condensa {
template <typename C>
static condensa_status quantize_impl(const float* x_dev, uint64_t n, uint16_t* q_dev, float* dq_dev, void* stream) {
    if (n > kMaxElems) return CONDENSA_ERR_SIZE;
    if (n == 0) return CONDENSA_OK;
    if (q_dev == nullptr && dq_dev == nullptr) return CONDENSA_ERR_NULL;
    if (x_dev == nullptr) return CONDENSA_ERR_NULL;
    const bool vec = aligned16(x_dev) && (!dq_dev || aligned16(dq_dev)) &&
                     (!q_dev || (reinterpret_cast<uintptr_t>(q_dev) & 7u) == 0);
    constexpr int QT = kQuantThreads;
    const u64 blocks = (n + QT * 4 - 1) / (QT * 4);           // x QT threads stays below 2^32 for n <= kMaxElems
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (!dq_dev && aligned16(x_dev) && aligned16(q_dev))
        hipLaunchKernelGGL((k_quantize_codes<QT, C>), dim3(static_cast<unsigned>((n + QT * 8 - 1) / (QT * 8))), dim3(QT), 0, st, x_dev, n, q_dev);
    else if (vec) hipLaunchKernelGGL((k_quantize<true, QT, C>), dim3(static_cast<unsigned>(blocks)), dim3(QT), 0, st, x_dev, n, q_dev, dq_dev);
    else     hipLaunchKernelGGL((k_quantize<false, QT, C>), dim3(static_cast<unsigned>(blocks)), dim3(QT), 0, st, x_dev, n, q_dev, dq_dev);
    CONDENSA_LAUNCH_CHECK();
    return CONDENSA_OK;
}

template <typename C>
static condensa_status dequantize_impl(const uint16_t* q_dev, uint64_t n, float* dq_dev, void* stream) {
    if (n > kMaxElems) return CONDENSA_ERR_SIZE;
    if (n == 0) return CONDENSA_OK;
    if (dq_dev == nullptr || q_dev == nullptr) return CONDENSA_ERR_NULL;
    const bool vec = aligned16(dq_dev) && (reinterpret_cast<uintptr_t>(q_dev) & 7u) == 0;
    constexpr int QT = kQuantThreads;
    const u64 blocks = (n + QT * 4 - 1) / (QT * 4);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (aligned16(q_dev) && aligned16(dq_dev))
        hipLaunchKernelGGL((k_dequantize_wide<QT, C>), dim3(static_cast<unsigned>((n + QT * 8 - 1) / (QT * 8))), dim3(QT), 0, st, q_dev, n, dq_dev);
    else if (vec) hipLaunchKernelGGL((k_dequantize<true, QT, C>), dim3(static_cast<unsigned>(blocks)), dim3(QT), 0, st, q_dev, n, dq_dev);
    else     hipLaunchKernelGGL((k_dequantize<false, QT, C>), dim3(static_cast<unsigned>(blocks)), dim3(QT), 0, st, q_dev, n, dq_dev);
    CONDENSA_LAUNCH_CHECK();
    return CONDENSA_OK;
}
template <typename C>
static condensa_status quantize8_impl(const float* x_dev, uint64_t n, uint8_t* q_dev, float* dq_dev, void* stream) {
    if (n > kMaxElems) return CONDENSA_ERR_SIZE;
    if (n == 0) return CONDENSA_OK;
    if (q_dev == nullptr && dq_dev == nullptr) return CONDENSA_ERR_NULL;
    if (x_dev == nullptr) return CONDENSA_ERR_NULL;
    const bool vec = aligned16(x_dev) && (!dq_dev || aligned16(dq_dev)) &&
                     (!q_dev || (reinterpret_cast<uintptr_t>(q_dev) & 3u) == 0);
    constexpr int QT = kQuantThreads;
    const u64 blocks = (n + QT * 4 - 1) / (QT * 4);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (!dq_dev && aligned16(x_dev) && aligned16(q_dev))
        hipLaunchKernelGGL((k_quantize8_codes<QT, C>), dim3(static_cast<unsigned>((n + QT * 16 - 1) / (QT * 16))), dim3(QT), 0, st, x_dev, n, q_dev);
    else if (vec) hipLaunchKernelGGL((k_quantize8<true, QT, C>), dim3(static_cast<unsigned>(blocks)), dim3(QT), 0, st, x_dev, n, q_dev, dq_dev);
    else     hipLaunchKernelGGL((k_quantize8<false, QT, C>), dim3(static_cast<unsigned>(blocks)), dim3(QT), 0, st, x_dev, n, q_dev, dq_dev);
    CONDENSA_LAUNCH_CHECK();
    return CONDENSA_OK;
}

template <typename C>
static condensa_status dequantize8_impl(const uint8_t* q_dev, uint64_t n, float* dq_dev, void* stream) {
    if (n > kMaxElems) return CONDENSA_ERR_SIZE;
    if (n == 0) return CONDENSA_OK;
    if (dq_dev == nullptr || q_dev == nullptr) return CONDENSA_ERR_NULL;
    const bool vec = aligned16(dq_dev) && (reinterpret_cast<uintptr_t>(q_dev) & 3u) == 0;
    constexpr int QT = kQuantThreads;
    const u64 blocks = (n + QT * 4 - 1) / (QT * 4);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (aligned16(q_dev) && aligned16(dq_dev))
        hipLaunchKernelGGL((k_dequantize8_wide<QT, C>), dim3(static_cast<unsigned>((n + QT * 16 - 1) / (QT * 16))), dim3(QT), 0, st, q_dev, n, dq_dev);
    else if (vec) hipLaunchKernelGGL((k_dequantize8<true, QT, C>), dim3(static_cast<unsigned>(blocks)), dim3(QT), 0, st, q_dev, n, dq_dev);
    else     hipLaunchKernelGGL((k_dequantize8<false, QT, C>), dim3(static_cast<unsigned>(blocks)), dim3(QT), 0, st, q_dev, n, dq_dev);
    CONDENSA_LAUNCH_CHECK();
    return CONDENSA_OK;
}
}  // namespace condensa

extern "C" {

condensa_status condensa_quantize_fp8(const float* x_dev, uint64_t n, int format, uint8_t* q_dev, float* dq_dev,
                                      void* stream) {
    if (format == CONDENSA_FP8_E4M3) return quantize8_impl<CodecE4M3>(x_dev, n, q_dev, dq_dev, stream);
    if (format == CONDENSA_FP8_E5M2) return quantize8_impl<CodecE5M2>(x_dev, n, q_dev, dq_dev, stream);
    return CONDENSA_ERR_ARG;
}

condensa_status condensa_dequantize_fp8(const uint8_t* q_dev, uint64_t n, int format, float* dq_dev, void* stream) {
    if (format == CONDENSA_FP8_E4M3) return dequantize8_impl<CodecE4M3>(q_dev, n, dq_dev, stream);
    if (format == CONDENSA_FP8_E5M2) return dequantize8_impl<CodecE5M2>(q_dev, n, dq_dev, stream);
    return CONDENSA_ERR_ARG;
}

condensa_status condensa_quantize(const float* x_dev, uint64_t n, uint16_t* q_dev, float* dq_dev, void* stream) {
    return quantize_impl<CodecF16>(x_dev, n, q_dev, dq_dev, stream);
}

condensa_status condensa_dequantize(const uint16_t* q_dev, uint64_t n, float* dq_dev, void* stream) {
    return dequantize_impl<CodecF16>(q_dev, n, dq_dev, stream);
}

condensa_status condensa_quantize_bf16(const float* x_dev, uint64_t n, uint16_t* q_dev, float* dq_dev, void* stream) {
    return quantize_impl<CodecBF16>(x_dev, n, q_dev, dq_dev, stream);
}

condensa_status condensa_dequantize_bf16(const uint16_t* q_dev, uint64_t n, float* dq_dev, void* stream) {
    return dequantize_impl<CodecBF16>(q_dev, n, dq_dev, stream);
}

condensa_status condensa_profile_read(int phase, double* total_ms, uint64_t* intervals) {
    if (phase < 0 || phase >= CONDENSA_PHASE_COUNT) return CONDENSA_ERR_ARG;
    if (total_ms == nullptr || intervals == nullptr) return CONDENSA_ERR_NULL;
    std::lock_guard<std::mutex> lock(g_prof_mu);
    for (Interval& iv : g_intervals) {
        CONDENSA_HIP(hipEventSynchronize(iv.b));
        float ms = 0.0f;
        CONDENSA_HIP(hipEventElapsedTime(&ms, iv.a, iv.b));
        g_phase_ms[iv.phase] += ms;
        g_phase_n[iv.phase] += 1;
        g_event_pool.push_back(iv.a);
        g_event_pool.push_back(iv.b);
    }
    g_intervals.clear();
    *total_ms = g_phase_ms[phase];
    *intervals = g_phase_n[phase];
    return CONDENSA_OK;
}

condensa_status condensa_profile_reset(void) {
    std::lock_guard<std::mutex> lock(g_prof_mu);
    for (Interval& iv : g_intervals) {
        (void)hipEventSynchronize(iv.b);
        g_event_pool.push_back(iv.a);
        g_event_pool.push_back(iv.b);
    }
    g_intervals.clear();
    for (int i = 0; i < CONDENSA_PHASE_COUNT; ++i) { g_phase_ms[i] = 0.0; g_phase_n[i] = 0; }
    return CONDENSA_OK;
}

condensa_status condensa_lc_sgd_step(const condensa_tensor* tensors, int n_tensors, const float* const* grad_loss,
                                     const float* const* theta, const float* const* lambda,
                                     float* const* momentum_buf, float mu, float lr, float momentum,
                                     void* workspace_dev, size_t workspace_bytes, void* stream,
                                     const condensa_config* config) {
    Config cfg;
    condensa_status rc = resolve_config(config, &cfg);
    if (rc != CONDENSA_OK) return rc;
    if (n_tensors > 0 && (!grad_loss || !theta || !lambda || !momentum_buf)) return CONDENSA_ERR_NULL;
    if (!(mu >= 0.0f) || !std::isfinite(mu) || !std::isfinite(lr) || !std::isfinite(momentum)) return CONDENSA_ERR_DENSITY;
    HostArena arena;
    Tables tb;
    rc = build_tensor_table(tensors, n_tensors, &tb, arena);
    if (rc != CONDENSA_OK) return rc;
    const Layout L = make_layout(CONDENSA_OP_LC_SGD_STEP, tb.N, 0, n_tensors, 1, CONDENSA_SCOPE_GLOBAL, cfg);
    std::vector<OutDesc> out(static_cast<size_t>(n_tensors > 0 ? n_tensors : 1), OutDesc{});
    std::vector<ByteRange> ranges;
    ranges.reserve(static_cast<size_t>(n_tensors) * 5 + 1);
    bool vec = tb.vec;
    for (int t = 0; t < n_tensors; ++t) {
        TensorDesc& d = tb.td[t];
        if (d.n == 0) continue;
        if (!grad_loss[t] || !theta[t] || !lambda[t] || !momentum_buf[t]) return CONDENSA_ERR_NULL;
        d.grad = const_cast<float*>(grad_loss[t]);
        d.lam = lambda[t];
        d.lam_out = momentum_buf[t];
        out[t].theta = const_cast<float*>(theta[t]);
        const void* ptrs[5] = {d.w, d.lam_out, d.grad, d.lam, out[t].theta};
        for (int i = 0; i < 5; ++i) {
            if (!aligned16(ptrs[i])) vec = false;
            ranges.push_back(byte_range(ptrs[i], d.n * 4, i < 2));     // the weights and the momentum buffer are written
        }
    }
    ranges.push_back(byte_range(workspace_dev, workspace_bytes < L.total ? workspace_bytes : L.total, true));
    if (ranges_conflict(ranges.data(), ranges.size())) return CONDENSA_ERR_ARG;
    rc = check_workspace(workspace_dev, workspace_bytes, L);
    if (rc != CONDENSA_OK) return rc;
    std::vector<char> up(L.upload_bytes, 0);
    std::memcpy(up.data() + L.td, tb.td, static_cast<size_t>(tb.n_td) * sizeof(TensorDesc));
    std::memcpy(up.data() + L.out, out.data(), out.size() * sizeof(OutDesc));
    hipStream_t st = static_cast<hipStream_t>(stream);
    rc = stage_upload(workspace_dev, up.data(), L.upload_bytes, st);
    if (rc != CONDENSA_OK) return rc;
    hipLaunchKernelGGL(k_prepare, dim3(fill_grid(L.zero_bytes / 8)), dim3(kBlock), 0, st,
                       at<u64>(workspace_dev, L.zero_begin), static_cast<u64>(L.zero_bytes / 8),
                       at<TensorDesc>(workspace_dev, L.td), n_tensors, at<u32>(workspace_dev, L.chunk_map), tb.n_chunks);
    CONDENSA_LAUNCH_CHECK();
    if (tb.n_chunks == 0) return CONDENSA_OK;
    DataArgs a{};
    a.td = at<TensorDesc>(workspace_dev, L.td);
    a.chunk_map = at<u32>(workspace_dev, L.chunk_map);
    a.n_chunks = tb.n_chunks;
    a.N = tb.N;
    a.n_tensors = n_tensors;
    a.mu = mu;
    PhaseTimer timer(CONDENSA_PHASE_APPLY, st, cfg);
    const OutDesc* od = at<OutDesc>(workspace_dev, L.out);
    const unsigned grid = static_cast<unsigned>(tb.n_chunks * (kChunk / 256));
    if (vec) hipLaunchKernelGGL((k_lc_sgd<true>), dim3(grid), dim3(64), 0, st, a, od, lr, momentum);
    else     hipLaunchKernelGGL((k_lc_sgd<false>), dim3(grid), dim3(64), 0, st, a, od, lr, momentum);
    CONDENSA_LAUNCH_CHECK();
    return CONDENSA_OK;
}

float condensa_mu_schedule(double mu0, double a, int j) { return static_cast<float>(mu0 * std::pow(a, static_cast<double>(j))); }

condensa_status condensa_thin(const float* w_dev, const int64_t* shape, int ndim, const int32_t* keep_out_dev,
                              int64_t n_keep_out, int64_t keep_out_offset, const int32_t* keep_in_dev,
                              int64_t n_keep_in, int64_t keep_in_offset, float* out_dev, void* stream) {
    if (shape == nullptr) return CONDENSA_ERR_NULL;
    if (ndim < 2 || ndim > 4) return CONDENSA_ERR_SHAPE;
    u64 ksize = 1;
    for (int i = 0; i < ndim; ++i) {
        if (shape[i] < 0 || shape[i] > 0x7FFFFFFFll) return CONDENSA_ERR_SHAPE;
        if (i >= 2) ksize *= static_cast<u64>(shape[i]);
    }
    const u64 c_out = static_cast<u64>(shape[0]), c_in = static_cast<u64>(shape[1]);
    if (n_keep_out < 0 || n_keep_in < 0) return CONDENSA_ERR_SIZE;
    const u64 n_out = keep_out_dev ? static_cast<u64>(n_keep_out) : c_out;
    const u64 n_in = keep_in_dev ? static_cast<u64>(n_keep_in) : c_in;
    if (n_out > 0x7FFFFFFFull || n_in > 0x7FFFFFFFull || ksize > 0x7FFFFFFFull) return CONDENSA_ERR_SIZE;
    const u64 total = n_out * n_in * ksize;
    if (total > kMaxElems) return CONDENSA_ERR_SIZE;
    if (total == 0) return CONDENSA_OK;
    if (w_dev == nullptr || out_dev == nullptr) return CONDENSA_ERR_NULL;
    {
        ByteRange r[4] = {byte_range(w_dev, c_out * c_in * ksize * 4, false), byte_range(out_dev, total * 4, true),
                          byte_range(keep_out_dev, keep_out_dev ? n_out * 4 : 0, false),
                          byte_range(keep_in_dev, keep_in_dev ? n_in * 4 : 0, false)};
        if (ranges_conflict(r, 4)) return CONDENSA_ERR_ARG;
    }
    u64 blocks = (total + kBlock - 1) / kBlock;
    if (blocks > 256 * 32) blocks = 256 * 32;
    hipLaunchKernelGGL(k_thin, dim3(static_cast<unsigned>(blocks)), dim3(kBlock), 0, static_cast<hipStream_t>(stream),
                       w_dev, c_out, c_in, ksize, keep_out_dev, n_out, keep_out_offset, keep_in_dev, n_in,
                       keep_in_offset, out_dev);
    CONDENSA_LAUNCH_CHECK();
    return CONDENSA_OK;
}

condensa_status condensa_set_option(int option, int64_t value) {
    if (option < 0 || option >= CONDENSA_OPT_COUNT) return CONDENSA_ERR_ARG;
    return set_default_option(option, value);
    return CONDENSA_OK;
}

int64_t condensa_get_option(int option) {
    if (option < 0 || option >= CONDENSA_OPT_COUNT) return -1;
    Config c;
    resolve_config(nullptr, &c);
    return c[option];
}

const char* condensa_status_string(condensa_status s) {
    switch (s) {
        case CONDENSA_OK: return "ok";
        case CONDENSA_ERR_NULL: return "required pointer is NULL";
        case CONDENSA_ERR_SIZE: return "count or size out of range";
        case CONDENSA_ERR_DENSITY: return "density outside [0,1], or mu not finite and positive";
        case CONDENSA_ERR_SHAPE: return "tensor shape not valid for this operator";
        case CONDENSA_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case CONDENSA_ERR_ARG: return "invalid scope, option or aliasing";
        case CONDENSA_ERR_HIP: return "HIP runtime call failed";
        default: return "unknown status";
    }
}

int condensa_last_hip_error(void) { return g_last_hip_error.load(); }

uint64_t condensa_launch_count(void) { return g_launches.load(); }

int condensa_version(void) { return 200; }

}  // extern "C"
