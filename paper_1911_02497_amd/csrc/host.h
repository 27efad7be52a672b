// Host-side plumbing shared by the entry points: status bookkeeping, per-call configuration, the pinned
// staging ring that carries the small per-call tables to the device, buffer-overlap checks, workspace carving.
#pragma once
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstring>
#include <mutex>
#include <vector>

#include "common.h"
#include "k_select.h"

namespace condensa {

extern std::atomic<int> g_last_hip_error;
extern std::atomic<uint64_t> g_launches;        // kernels enqueued since the library was loaded (diagnostic)

// The knobs of one call, resolved once at the entry point: the caller's condensa_config, or the
// process-wide defaults when it passes NULL.  Everything below the entry point reads this copy only.
struct Config {
    int64_t v[CONDENSA_OPT_COUNT];
    int64_t operator[](int option) const { return v[option]; }
};
condensa_status resolve_config(const condensa_config* c, Config* out);   // CONDENSA_ERR_ARG for invalid values
condensa_status set_default_option(int option, int64_t value);

#define CONDENSA_HIP(expr)                                                      \
    do {                                                                        \
        hipError_t err__ = (expr);                                              \
        if (err__ != hipSuccess) {                                              \
            ::condensa::g_last_hip_error.store(static_cast<int>(err__));        \
            return CONDENSA_ERR_HIP;                                            \
        }                                                                       \
    } while (0)

#define CONDENSA_LAUNCH_CHECK()                                                 \
    do {                                                                        \
        ::condensa::g_launches.fetch_add(1, std::memory_order_relaxed);         \
        CONDENSA_HIP(hipGetLastError());                                        \
    } while (0)

inline size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// k = llround(density * n) clamped to [0, n]; the product is taken in binary64.
inline u64 kept_count(double density, u64 n) {
    const double x = density * static_cast<double>(n);
    const long long r = std::llround(x);
    if (r < 0) return 0;
    if (static_cast<u64>(r) > n) return n;
    return static_cast<u64>(r);
}

inline bool density_ok(double d) { return d >= 0.0 && d <= 1.0; }   // false for NaN

// Copies `bytes` of host data to device memory on `stream` through a pinned ring, so the caller's
// tables can be released as soon as the entry point returns and the call never waits for the GPU
// unless all ring slots are still in flight.
condensa_status stage_upload(void* dst_dev, const void* src_host, size_t bytes, hipStream_t stream);

// Phase timing: records an event pair around the launches made while the object lives, when the call's
// profile mask asks for that phase.  The pair belongs to the object until both events are recorded;
// only then is it handed to the list that condensa_profile_read drains.
class PhaseTimer {
public:
    PhaseTimer(int phase, hipStream_t stream, const Config& cfg);
    ~PhaseTimer();
    PhaseTimer(const PhaseTimer&) = delete;
    PhaseTimer& operator=(const PhaseTimer&) = delete;
private:
    hipEvent_t a_ = nullptr, b_ = nullptr;
    int phase_;
    hipStream_t stream_;
};

// Byte ranges of the buffers of one call.  A call is rejected when an output overlaps any other range.
// An input that the call also writes in place (theta == w, lambda updated in place) is entered once, as
// an output.
struct ByteRange {
    uintptr_t begin, end;
    bool written;
};
inline ByteRange byte_range(const void* p, u64 bytes, bool written) {
    const uintptr_t b = reinterpret_cast<uintptr_t>(p);
    return ByteRange{b, b + static_cast<uintptr_t>(p ? bytes : 0), written};
}
// Sorts `r` by start address; true when some written range overlaps another range.
inline bool ranges_conflict(ByteRange* r, size_t n) {
    std::sort(r, r + n, [](const ByteRange& x, const ByteRange& y) { return x.begin < y.begin; });
    uintptr_t end_any = 0, end_written = 0;          // furthest end among the ranges seen so far
    for (size_t i = 0; i < n; ++i) {
        if (r[i].begin == r[i].end) continue;        // empty
        if (r[i].written ? r[i].begin < end_any : r[i].begin < end_written) return true;
        if (r[i].end > end_any) end_any = r[i].end;
        if (r[i].written && r[i].end > end_written) end_written = r[i].end;
    }
    return false;
}

// Element count of a tensor; false if the descriptor is malformed.
inline bool tensor_elems(const condensa_tensor& t, u64* n) {
    if (t.ndim < 1 || t.ndim > 4 || t.reserved != 0) return false;
    u64 p = 1;
    for (int i = 0; i < t.ndim; ++i) {
        if (t.shape[i] < 0) return false;
        const u64 d = static_cast<u64>(t.shape[i]);
        if (d != 0 && p > kMaxElems / d) return false;   // cap at kMaxElems
        p *= d;
    }
    *n = p;
    return true;
}

// Carving of the caller's workspace.  Offsets are multiples of 256 bytes.
constexpr unsigned kStructLevels = 6;     // radix levels of a 63-bit structure key (11+11+11+10+10+10 bits)

struct Layout {
    size_t td = 0, out = 0, slots = 0, upload_bytes = 0;   // [td | out | slots] is uploaded in one copy
    size_t zero_begin = 0, zero_bytes = 0;                 // [ctl | hist0 | histx] is cleared by one kernel
    size_t ctl = 0, hist0 = 0, histx = 0, histc = 0, seg = 0;   // histc: coarse sums; seg: window-path segment counters
    size_t tiecnt = 0, tiehit = 0, chunk_map = 0;
    size_t tl_cnt = 0, tl_key = 0, tl_idx = 0;              // short lists of the keys that reach the last radix level's bins
    u64 small_cap = 0;                                      // small calls: entries of the one list that replaces them (0: not a small call)
    size_t skeys = 0, sblock = 0, smask = 0;                // structure keys, per-block kept counts, keep flags
    size_t sample = 0, cand_key = 0, cand_idx = 0;          // window path
    size_t cand_w = 0, cand_lam = 0;                        // inputs of the candidates (fused sweep)
    size_t sorted_windows = 0;                              // several densities: the windows in sweep order
    u64 sample_cap = 0, cand_cap = 0;
    size_t total = 0;
    u64 max_chunks = 0, max_schunks = 0;
    int n_groups = 1, n_slots = 1;
};

Layout make_layout(int op, u64 total_elems, u64 n_structures, int n_tensors, int n_densities, int scope,
                   const Config& cfg, bool no_window = false);

}  // namespace condensa
