// Sampled-window selection: the exact k-th largest key with ONE sweep over the weights.
//
// A jittered, stratified sample of the keys is ranked exactly; the keys at two sample ranks around
// the expected position of the threshold bound a key window [lo, hi] that holds the true threshold
// unless the sample was unlucky.  One sweep over all weights then counts the keys above hi and
// compacts the (key, flat index) of the keys inside the window; the threshold and the tie rule are
// resolved exactly on that short candidate list.  A window that turns out not to hold the wanted
// rank (or a candidate list that overflows) is detected on the device and the ranking falls back to
// the radix levels over the weights, so the result never depends on the sample.
// Section 3.1: the magnitude threshold that realises a given sparsity; several target sparsities of one
// search (Results: up to 10 samples per search) are served by the same sweep.
#pragma once
#include "host.h"
#include "k_select.h"

namespace condensa {

constexpr int kSampleUnit = 4;         // consecutive elements read at one sample position
constexpr int kArrayWords = 4 * kBins;  // LDS histogram words of the array kernels (32 KB)
constexpr int kArrayBatchMax = 8;      // at most this many rankings per pass over a key array
constexpr u32 kNoKey = 0xFFFFFFFFu;    // marks sample entries that fell past the end of a tensor
constexpr int kArrayThreads = 1024;     // workgroup of the array kernels: wide, so that few workgroups flush their
                                       // LDS histograms with (slow, memory-side) global atomics
constexpr int kSegs = 1024;            // candidate list segments / counter sets (see k_window_sweep)

// The one-density fused sweep stores a candidate's tensor above its flat index, so that the fix-up pass need not
// search the tensor table for it (flat indices stay below 2^44, tensor numbers below 2^20: checked by the host).
constexpr int kCandTensorShift = 44;
static_assert(CONDENSA_MAX_TENSORS <= (1 << (64 - kCandTensorShift)), "tensor numbers must fit above the flat index");
__device__ inline u64 cand_pack(u64 flat, int t) { return flat | (static_cast<u64>(t) << kCandTensorShift); }
__device__ inline u64 cand_flat(u64 packed) { return packed & ((static_cast<u64>(1) << kCandTensorShift) - 1); }
__device__ inline int cand_tensor(u64 packed) { return static_cast<int>(packed >> kCandTensorShift); }

struct SortedWindows;

struct WindowArgs {
    u32* sample;           // [n_units * kSampleUnit]
    u32* cand_key;         // [cand_cap]
    u64* cand_idx;         // [cand_cap] flat indices (fused sweep: cand_pack)
    Slot* wslots;          // [2J] boundary rankings, later [J] index rankings
    u64* seg_cnt;          // [kSegs] candidates appended to each segment (may exceed seg_cap)
    u64* seg_region;       // [kMaxJ + 1][kSegs] keys per region (region i: i windows have an upper bound >= key)
    u64 seg_cap;           // entries per segment
    u32 n_segs;            // segments in use
    u64 n_units;
    u64 stride;            // sample positions are one per stride of quads
    u64 cand_cap;
    int margin16;
    u64* tie_list;         // [tie_cap] flat indices of the candidates equal to the threshold (one density)
    u64 tie_cap;
    float* cand_w;         // [cand_cap] fused sweep: weight of each candidate
    float* cand_lam;       // [cand_cap] fused sweep: multiplier of each candidate (L-C step)
    const OutDesc* out;    // fused sweep: output table
    struct SortedWindows* sorted;   // several densities: the windows in sweep order, written by k_window_sort
    u64* hist_main;        // histograms of the candidate rankings
    u64* hist_aux;         // histograms of the sample's boundary rankings, later of the index rankings
    u64* hist_shared0;     // level 0 of the sample, shared by its boundary rankings
};

struct ArrayArgs {
    const u32* keys;       // sample or candidate keys
    const u64* idx;        // candidate flat indices (index ranking only)
    u64 n_host;            // number of entries (plain array)
    const u64* seg_cnt;    // NULL: plain array; else the array is n_segs segments of seg_cap entries
    u64 seg_cap;
    u32 n_segs;
    u64 N;                 // index ranking: the ranked key is N - 1 - idx
    Slot* slots;
    u64* hist;             // [n_slots][kBins]
    u64* shared0;          // NULL, or: all rankings have the same filter and no prefix at level 0, count once here
    const u32* gate;       // NULL, or skip the kernel when *gate == 0
    int n_slots;
    int key_bits;
    int merged;            // 1: hist holds one histogram per level and ranking ([level][n_slots]) and every level
                           // kernel folds in the previous level itself (wave_enter_level); 0: k_scan_level in between
    u64* hist_base;        // merged form: first histogram of the workspace and the coarse sums of all of them
    u64* coarse;
};

__device__ inline u64* array_hist(const ArrayArgs& a, int level, int slot) {
    return a.hist + (a.merged ? static_cast<u64>(level) * a.n_slots + slot : static_cast<u64>(slot)) * kBins;
}

__device__ inline u32 mix32(u32 x) {
    x ^= x >> 16; x *= 0x9E3779B1u;
    x ^= x >> 13; x *= 0x85EBCA77u;
    x ^= x >> 16;
    return x;
}

// ---- sample -----------------------------------------------------------------------------------------
template <bool LC, bool VEC>
__global__ __launch_bounds__(kBlock) void k_sample(DataArgs a, WindowArgs w) {
    __shared__ u32 s_valid;
    const int tid = threadIdx.x;
    if (tid == 0) s_valid = 0;
    __syncthreads();
    const u64 u = static_cast<u64>(blockIdx.x) * kBlock + tid;
    u32 n_valid = 0;
    if (u < w.n_units) {
        const u64 jitter = (w.stride > 1) ? static_cast<u64>(mix32(static_cast<u32>(u) ^ static_cast<u32>(u >> 32))) % w.stride : 0;
        const u64 p = u * w.stride + jitter;             // quad position in chunk space
        const u64 c = p / (kChunk / 4);
        const u64 q = p % (kChunk / 4);
        u32 key[4] = {kNoKey, kNoKey, kNoKey, kNoKey};
        if (c < a.n_chunks) {
            const int t = static_cast<int>(a.chunk_map[c]);
            const TensorDesc& td = a.td[t];
            const u64 e0 = (c - td.chunk_start) * kChunk + q * 4;
            if (e0 < td.n) {
                float v[4];
                load4<VEC>(td.w, e0, td.n, v);
                if (LC) {
                    float l[4];
                    load4<VEC>(td.lam, e0, td.n, l);
#pragma unroll
                    for (int k = 0; k < 4; ++k) v[k] = lc_shift(v[k], l[k], a.mu);
                }
#pragma unroll
                for (int k = 0; k < 4; ++k)
                    if (e0 + k < td.n) { key[k] = mag_key(v[k]); ++n_valid; }
            }
        }
        *reinterpret_cast<uint4*>(w.sample + u * 4) = make_uint4(key[0], key[1], key[2], key[3]);
    }
    if (n_valid) atomicAdd(&s_valid, n_valid);
    __syncthreads();
    if (tid == 0 && s_valid) atomicAdd(reinterpret_cast<unsigned long long*>(&a.ctl->sample_count), static_cast<unsigned long long>(s_valid));
}

// One density: the sample and the level-0 histogram of its keys in one kernel (the boundary rankings share
// that level), so the sample is not read back for it.  Few wide workgroups: each flushes its LDS counts with
// global atomics, which are slow on one address.
constexpr int kSampleHistThreads = 1024;
template <bool LC, bool VEC>
__global__ __launch_bounds__(kSampleHistThreads) void k_sample_hist(DataArgs a, WindowArgs w, ArrayArgs ar) {
    __shared__ u32 s_hist[kBins];
    const int tid = threadIdx.x;
    const Level L0 = level_of(31, 0);
    for (int i = tid; i < kBins; i += kSampleHistThreads) s_hist[i] = 0;
    __syncthreads();
    for (u64 u = static_cast<u64>(blockIdx.x) * kSampleHistThreads + tid; u < w.n_units; u += static_cast<u64>(gridDim.x) * kSampleHistThreads) {
        const u64 jitter = (w.stride > 1) ? static_cast<u64>(mix32(static_cast<u32>(u) ^ static_cast<u32>(u >> 32))) % w.stride : 0;
        const u64 p = u * w.stride + jitter;             // quad position in chunk space
        const u64 c = p / (kChunk / 4);
        const u64 q = p % (kChunk / 4);
        u32 key[4] = {kNoKey, kNoKey, kNoKey, kNoKey};
        if (c < a.n_chunks) {
            const int t = static_cast<int>(a.chunk_map[c]);
            const TensorDesc& td = a.td[t];
            const u64 e0 = (c - td.chunk_start) * kChunk + q * 4;
            if (e0 < td.n) {
                float v[4];
                load4<VEC>(td.w, e0, td.n, v);
                if (LC) {
                    float l[4];
                    load4<VEC>(td.lam, e0, td.n, l);
#pragma unroll
                    for (int k = 0; k < 4; ++k) v[k] = lc_shift(v[k], l[k], a.mu);
                }
#pragma unroll
                for (int k = 0; k < 4; ++k)
                    if (e0 + k < td.n) {
                        key[k] = mag_key(v[k]);
                        atomicAdd(&s_hist[key[k] >> L0.shift], 1u);
                    }
            }
        }
        *reinterpret_cast<uint4*>(w.sample + u * 4) = make_uint4(key[0], key[1], key[2], key[3]);
    }
    __syncthreads();
    const int run = coarse_run(kBins);
    for (int i = tid; i < kBins; i += kSampleHistThreads) {
        const u32 v = s_hist[i];
        if (v) atomicAdd(reinterpret_cast<unsigned long long*>(ar.shared0 + i), static_cast<unsigned long long>(v));
    }
    if (tid < kCoarse) {
        u32 v = 0;
        for (int t = tid * run; t < (tid + 1) * run; ++t) v += s_hist[t];
        if (v) atomicAdd(reinterpret_cast<unsigned long long*>(coarse_of(ar.hist_base, ar.coarse, ar.shared0) + tid), static_cast<unsigned long long>(v));
    }
}

// Sample ranks that bound each density's threshold.  The number of sample keys above the true
// threshold is (close to) binomial; sample units of kSampleUnit neighbours may be correlated, so the
// standard deviation is taken as if every unit were one draw.
__global__ __launch_bounds__(kBlock) void k_window_ranks(DataArgs a, WindowArgs w) {
    const int j = threadIdx.x;
    if (j >= a.J) return;
    const Slot& main = a.slots[j];
    const u64 S = a.ctl->sample_count;
    Slot hi{}, lo{};
    hi.n = lo.n = S;
    hi.lo = lo.lo = 0;
    hi.hi = lo.hi = 0x7FFFFFFFu;
    hi.state = lo.state = kDone;
    hi.prefix = 0x7FFFFFFFu;                             // no upper bound
    lo.prefix = 0;                                       // no lower bound
    if (main.state == kSelecting && S > 0) {
        const double p = static_cast<double>(main.k) / static_cast<double>(main.n);
        const double ks = p * static_cast<double>(S);
        const double sd = sqrt(static_cast<double>(kSampleUnit) * static_cast<double>(S) * p * (1.0 - p));
        const double m = static_cast<double>(w.margin16) / 16.0 * sd + 2.0;
        const double rhi = floor(ks - m);
        const double rlo = ceil(ks + m) + 1.0;
        if (rhi >= 1.0) { hi.state = kSelecting; hi.prefix = 0; hi.remaining = static_cast<u64>(rhi); }
        if (rlo <= static_cast<double>(S)) { lo.state = kSelecting; lo.prefix = 0; lo.remaining = static_cast<u64>(rlo); }
    }
    w.wslots[2 * j] = hi;
    w.wslots[2 * j + 1] = lo;
}

// ---- histogram of one radix level over a key array -------------------------------------------------
// Entry i takes part in ranking j when its key lies in [slot.lo, slot.hi] and the ranked key (the key
// itself, or N - 1 - idx for the index ranking) matches the ranking's prefix.
template <bool IDX>
__global__ __launch_bounds__(kArrayThreads) void k_hist_array(ArrayArgs a, int level) {
    __shared__ u32 s_hist[kArrayWords];
    __shared__ u64 s_prefix[kArrayBatchMax];
    __shared__ u32 s_lo[kArrayBatchMax], s_hi[kArrayBatchMax], s_active[kArrayBatchMax];
    __shared__ u64 s_mprefix[2 * kMaxJ + 1];   // merged form: the rankings' state on entering this level
    __shared__ u32 s_mactive[2 * kMaxJ + 1];
    __shared__ u32 s_any;
    if (a.gate && *a.gate == 0) return;
    if (a.merged) {
        for (int j = static_cast<int>(threadIdx.x) >> 6; j < a.n_slots; j += kArrayThreads / 64) {
            const u64* prev = (level == 1 && a.shared0) ? a.shared0 : array_hist(a, level > 0 ? level - 1 : 0, j);
            const SlotStep e = wave_enter_level(a.slots[j], level, a.key_bits, prev, coarse_of(a.hist_base, a.coarse, prev));
            if ((threadIdx.x & 63) == 0) {
                s_mprefix[j] = e.prefix;
                s_mactive[j] = (e.state == kSelecting && static_cast<u32>(level) >= a.slots[j].level_begin) ? 1u : 0u;
                if (blockIdx.x == 0 && level > 0) a.slots[j].step[level & 1] = e;
            }
        }
        __syncthreads();
    }
    const int nt = static_cast<int>(blockDim.x);
    const Level L = level_of(a.key_bits, level);
    const int nb = 1 << L.bits;
    const int tid = threadIdx.x;
    const bool share = (level == 0 && a.shared0 != nullptr);
    int batch = kArrayWords / nb;
    if (batch > kArrayBatchMax) batch = kArrayBatchMax;
    const int n_slots = share ? 1 : a.n_slots;
    for (int j0 = 0; j0 < n_slots; j0 += batch) {
        const int nj = (n_slots - j0 < batch) ? n_slots - j0 : batch;
        __syncthreads();
        if (tid == 0) s_any = 0;
        __syncthreads();
        if (share) {
            // one count serves every ranking: active when any of them still selects
            if (tid < a.n_slots && a.slots[tid].state == kSelecting && a.slots[tid].level_begin == 0) s_any = 1;
            if (tid == 0) {
                s_prefix[0] = 0;
                s_lo[0] = static_cast<u32>(a.slots[0].lo);
                s_hi[0] = static_cast<u32>(a.slots[0].hi);
                s_active[0] = 1;
            }
        } else if (tid < nj) {
            const Slot& s = a.slots[j0 + tid];
            s_prefix[tid] = a.merged ? s_mprefix[j0 + tid] : s.prefix;
            s_lo[tid] = static_cast<u32>(s.lo);
            s_hi[tid] = static_cast<u32>(s.hi);
            const bool on = a.merged ? s_mactive[j0 + tid] != 0
                                     : (s.state == kSelecting && static_cast<u32>(level) >= s.level_begin);
            s_active[tid] = on ? 1u : 0u;
            if (on) s_any = 1;
        }
        __syncthreads();
        if (!s_any) continue;                            // uniform: nothing to count in this batch
        // Keys of a sample or of a narrow window crowd into a few bins; spare LDS holds private copies
        // of the histograms, chosen by lane, so that fewer lanes of a wavefront hit one address.
        int copies = 1;
        while (copies < 8 && 2 * copies * nj * nb <= kArrayWords) copies *= 2;
        const int words = nj * nb;
        for (int i = tid; i < copies * words; i += nt) s_hist[i] = 0;
        __syncthreads();
        u32* my_hist = s_hist + (tid & (copies - 1)) * words;
        // entries are fetched eight at a time so that their loads overlap (the loop is latency bound)
        constexpr int kUnroll = 8;
        auto count_entry = [&](u32 ck, u64 ix) {
            const u64 rk = IDX ? (a.N - 1 - ix) : static_cast<u64>(ck);
            const u32 digit = static_cast<u32>(rk >> L.shift) & (nb - 1);
            for (int j = 0; j < nj; ++j)
                if (s_active[j] && ck >= s_lo[j] && ck <= s_hi[j] && ((rk ^ s_prefix[j]) >> L.hi_shift) == 0)
                    atomicAdd(&my_hist[j * nb + digit], 1u);
        };
        if (a.seg_cnt) {
            // A workgroup owns every gridDim.x-th segment.  Four segments are read together, two entries of
            // each per thread and step: the segments are short (a thousand entries), and walking them one
            // after the other would pay one round trip for the count and one for the entries of each.
            constexpr int kSegBatch = 4, kPer = kUnroll / kSegBatch;
            for (u32 seg0 = blockIdx.x; seg0 < a.n_segs; seg0 += gridDim.x * kSegBatch) {
                u64 cnt[kSegBatch], first[kSegBatch], most = 0;
#pragma unroll
                for (int b = 0; b < kSegBatch; ++b) {
                    const u64 seg = static_cast<u64>(seg0) + static_cast<u64>(b) * gridDim.x;
                    u64 c = (seg < a.n_segs) ? a.seg_cnt[seg < a.n_segs ? seg : 0] : 0;
                    if (c > a.seg_cap) c = a.seg_cap;
                    cnt[b] = c;
                    first[b] = seg * a.seg_cap;
                    most = c > most ? c : most;
                }
                for (u64 i0 = tid; i0 < most; i0 += static_cast<u64>(nt) * kPer) {
                    u32 ck[kUnroll];
                    u64 ix[kUnroll];
#pragma unroll
                    for (int u = 0; u < kUnroll; ++u) {
                        const int b = u % kSegBatch;
                        const u64 i = i0 + static_cast<u64>(nt) * (u / kSegBatch);
                        ck[u] = (i < cnt[b]) ? a.keys[first[b] + i] : kNoKey;
                        ix[u] = (IDX && i < cnt[b]) ? a.idx[first[b] + i] : 0;
                    }
#pragma unroll
                    for (int u = 0; u < kUnroll; ++u)
                        if (i0 + static_cast<u64>(nt) * (u / kSegBatch) < cnt[u % kSegBatch]) count_entry(ck[u], ix[u]);
                }
            }
        } else {
            const u64 step = static_cast<u64>(gridDim.x) * nt;
            for (u64 i0 = static_cast<u64>(blockIdx.x) * nt + tid; i0 < a.n_host; i0 += step * kUnroll) {
                u32 ck[kUnroll];
                u64 ix[kUnroll];
#pragma unroll
                for (int u = 0; u < kUnroll; ++u) {
                    const u64 i = i0 + step * u;
                    ck[u] = (i < a.n_host) ? a.keys[i] : kNoKey;
                    ix[u] = (IDX && i < a.n_host) ? a.idx[i] : 0;
                }
#pragma unroll
                for (int u = 0; u < kUnroll; ++u)
                    if (i0 + step * u < a.n_host) count_entry(ck[u], ix[u]);
            }
        }
        __syncthreads();
        u64* dst = share ? a.shared0 : array_hist(a, level, j0);
        for (int i = tid; i < words; i += nt) {
            u32 v = 0;
            for (int cpy = 0; cpy < copies; ++cpy) v += s_hist[cpy * words + i];
            if (v) atomicAdd(reinterpret_cast<unsigned long long*>(dst + static_cast<u64>(i / nb) * kBins + (i % nb)),
                             static_cast<unsigned long long>(v));
        }
        if (a.merged) {                                  // the coarse sums of the same counts
            const int run = coarse_run(nb);
            for (int i = tid; i < nj * kCoarse; i += nt) {
                const int h = i / kCoarse, c = i % kCoarse;
                u32 v = 0;
                for (int t = c * run; t < (c + 1) * run && t < nb; ++t)
                    for (int cpy = 0; cpy < copies; ++cpy) v += s_hist[cpy * words + h * nb + t];
                if (v) atomicAdd(reinterpret_cast<unsigned long long*>(coarse_of(a.hist_base, a.coarse, dst + static_cast<u64>(h) * kBins) + c),
                                 static_cast<unsigned long long>(v));
            }
        }
    }
}

// ---- the one sweep over the weights -----------------------------------------------------------------
// Counters and the candidate list are split into segments chosen by the workgroup id: one global
// atomic address shared by ~10^5 workgroups serialises the whole sweep, a thousand addresses do not.
//
// Several densities: the windows of the active rankings are put in descending order of their upper
// bound.  For a key, i = number of windows whose upper bound is >= key places it in region i; the keys
// above the window at sorted position p are the regions 0..p, and the key is a candidate iff it is
// >= the smallest lower bound among the first i windows.  Region counts of a thread (at most 32 keys)
// are packed in 6-bit fields.

struct SortedWindows {
    u32 hi[kMaxJ];         // upper bounds, descending
    u32 minlo[kMaxJ];      // minlo[p] = smallest lower bound among sorted positions 0..p
    u32 slot[kMaxJ];       // ranking at each sorted position
    u32 n;                 // active rankings
};

// Deterministic order (upper bound descending, then lower bound descending, then ranking id); run by
// one thread -- at most kMaxJ entries.
__device__ inline void sort_windows(const Slot* slots, const Slot* wslots, int J, SortedWindows* out) {
    u32 hi[kMaxJ], lo[kMaxJ], id[kMaxJ];
    u32 n = 0;
    for (int j = 0; j < J; ++j) {
        if (slots[j].state != kSelecting) continue;
        const u32 h = static_cast<u32>(wslots[2 * j].prefix), l = static_cast<u32>(wslots[2 * j + 1].prefix);
        u32 p = n;
        while (p > 0 && (hi[p - 1] < h || (hi[p - 1] == h && lo[p - 1] < l))) {
            hi[p] = hi[p - 1]; lo[p] = lo[p - 1]; id[p] = id[p - 1];
            --p;
        }
        hi[p] = h; lo[p] = l; id[p] = static_cast<u32>(j);
        ++n;
    }
    u32 m = 0xFFFFFFFFu;
    for (u32 p = 0; p < n; ++p) {
        m = lo[p] < m ? lo[p] : m;
        out->hi[p] = hi[p];
        out->minlo[p] = m;
        out->slot[p] = id[p];
    }
    out->n = n;
}

// Runs once between the sample ranking and the sweep (one thread): ordering the windows inside every
// workgroup of the sweep, a chain of ~2J dependent global loads in one thread, cost the sweep more than
// its memory traffic.
__global__ void k_window_sort(DataArgs a, WindowArgs w) {
    if (threadIdx.x == 0 && blockIdx.x == 0) sort_windows(a.slots, w.wslots, a.J, w.sorted);
}

template <bool LC, bool VEC>
__global__ __launch_bounds__(kBlock) void k_window_sweep(DataArgs a, WindowArgs w) {
    __shared__ SortedWindows s_win;
    __shared__ u32 s_region[kMaxJ + 1];
    __shared__ u64 s_wave[kBlock / 64];
    __shared__ u64 s_base;
    const u64 c = blockIdx.x;
    if (c >= a.n_chunks) return;
    const int tid = threadIdx.x;
    if (tid < static_cast<int>(sizeof(SortedWindows) / sizeof(u32)))
        reinterpret_cast<u32*>(&s_win)[tid] = reinterpret_cast<const u32*>(w.sorted)[tid];
    if (tid <= kMaxJ) s_region[tid] = 0;
    __syncthreads();
    const int n = static_cast<int>(s_win.n);
    const int t = static_cast<int>(a.chunk_map[c]);
    const TensorDesc& td = a.td[t];
    const u64 base = (c - td.chunk_start) * kChunk;

    u32 key[kQuadsPerThread][4];
    u32 cmask = 0;
    u64 pk0 = 0, pk1 = 0;                 // 6-bit counts of regions 0..9 and 10..16
    const bool full = VEC && !LC && base + kChunk <= td.n;               // uniform: all loads first
    float4 wv[kQuadsPerThread];
    if (full) {
#pragma unroll
        for (int q = 0; q < kQuadsPerThread; ++q) wv[q] = ld4_stream(td.w + base + q * (kBlock * 4) + tid * 4);
    }
#pragma unroll
    for (int q = 0; q < kQuadsPerThread; ++q) {
        const u64 e0 = base + static_cast<u64>(q) * (kBlock * 4) + tid * 4;
        float v[4] = {0.f, 0.f, 0.f, 0.f};
        if (full) {
            v[0] = wv[q].x; v[1] = wv[q].y; v[2] = wv[q].z; v[3] = wv[q].w;
        } else if (e0 < td.n) {
            load4<VEC>(td.w, e0, td.n, v);
            if (LC) {
                float l[4];
                load4<VEC>(td.lam, e0, td.n, l);
#pragma unroll
                for (int k = 0; k < 4; ++k) v[k] = lc_shift(v[k], l[k], a.mu);
            }
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const u32 x = mag_key(v[k]);
            key[q][k] = x;
            if (e0 + k < td.n) {
                int i = 0;
                for (int p = 0; p < n; ++p) i += (s_win.hi[p] >= x) ? 1 : 0;
                if (i < 10) pk0 += static_cast<u64>(1) << (6 * i);
                else        pk1 += static_cast<u64>(1) << (6 * (i - 10));
                if (i > 0 && x >= s_win.minlo[i - 1]) cmask |= 1u << (q * 4 + k);
            }
        }
    }
    // region counts: wavefront sums, then one LDS and one global atomic per workgroup and region
    for (int r = 0; r <= n; ++r) {
        u32 sum = static_cast<u32>(r < 10 ? (pk0 >> (6 * r)) : (pk1 >> (6 * (r - 10)))) & 63u;
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) sum += __shfl_down(sum, d, 64);
        if ((tid & 63) == 0 && sum) atomicAdd(&s_region[r], sum);
    }
    // candidates: one reservation per workgroup, then every thread writes its own in order
    u64 total;
    const u64 off = block_excl_scan_u64(__popc(cmask), s_wave, &total);    // syncs the workgroup
    const u32 seg = static_cast<u32>(c % w.n_segs);
    if (tid <= n && s_region[tid])
        atomicAdd(reinterpret_cast<unsigned long long*>(&w.seg_region[static_cast<u64>(tid) * kSegs + seg]),
                  static_cast<unsigned long long>(s_region[tid]));
    if (total == 0) return;
    if (tid == 0)
        s_base = atomicAdd(reinterpret_cast<unsigned long long*>(&w.seg_cnt[seg]), static_cast<unsigned long long>(total));
    __syncthreads();
    if (cmask == 0) return;
    u64 pos = s_base + off;
    const u64 first = static_cast<u64>(seg) * w.seg_cap;
#pragma unroll
    for (int q = 0; q < kQuadsPerThread; ++q) {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            if (cmask & (1u << (q * 4 + k))) {
                if (pos < w.seg_cap) {
                    w.cand_key[first + pos] = key[q][k];
                    w.cand_idx[first + pos] = td.flat_start + base + static_cast<u64>(q) * (kBlock * 4) + tid * 4 + k;
                }
                ++pos;
            }
        }
    }
}

// Single-density form of the sweep: one wavefront per workgroup, 8 KB of input each (1024 elements
// with multipliers, 2048 without), so there is no workgroup barrier; the wavefront reserves its
// candidate slots with one atomic on its segment.  Workgroups that lie wholly inside their tensor (all
// but the last one of a tensor) issue every load before the first use, which keeps 4-8 loads per lane in
// flight; the ragged last workgroup takes the guarded path.
template <bool LC, bool VEC, int QUADS>
__global__ __launch_bounds__(64) void k_window_sweep_wave(DataArgs a, WindowArgs w) {
    constexpr int kWaveElems = 64 * 4 * QUADS;
    constexpr u32 kSub = kChunk / kWaveElems;
    const u64 c = blockIdx.x / kSub;
    const u32 sub = blockIdx.x % kSub;
    if (c >= a.n_chunks) return;
    const int lane = threadIdx.x;
    const int t = static_cast<int>(a.chunk_map[c]);
    const TensorDesc& td = a.td[t];
    const u64 base = (c - td.chunk_start) * kChunk + static_cast<u64>(sub) * kWaveElems;
    const u64 n = td.n;
    if (base >= n) return;
    if (a.slots[0].state != kSelecting) return;                         // nothing to count (k == 0)
    const u32 hi = static_cast<u32>(w.wslots[0].prefix);
    const u32 lo = static_cast<u32>(w.wslots[1].prefix);
    const u32 span = hi - lo;                                           // lo <= hi: x in [lo, hi] <=> x - lo <= span
    const float* __restrict__ wp = td.w;
    const float* __restrict__ lp = td.lam;

    u32 key[QUADS][4];
    u32 cmask = 0, above = 0;
    if (VEC && base + kWaveElems <= n) {                                // uniform over the wavefront
        float4 wv[QUADS], lv[QUADS];
#pragma unroll
        for (int q = 0; q < QUADS; ++q) {
            wv[q] = ld4_stream(wp + base + q * 256 + lane * 4);
            if (LC) lv[q] = ld4_stream(lp + base + q * 256 + lane * 4);
        }
#pragma unroll
        for (int q = 0; q < QUADS; ++q) {
            float v[4] = {wv[q].x, wv[q].y, wv[q].z, wv[q].w};
            if (LC) {
                const float l[4] = {lv[q].x, lv[q].y, lv[q].z, lv[q].w};
#pragma unroll
                for (int k = 0; k < 4; ++k) v[k] = lc_shift(v[k], l[k], a.mu);
            }
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const u32 x = mag_key(v[k]);
                key[q][k] = x;
                above += (x > hi) ? 1u : 0u;
                cmask |= ((x - lo <= span) ? 1u : 0u) << (q * 4 + k);
            }
        }
    } else {
#pragma unroll
        for (int q = 0; q < QUADS; ++q) {
            const u64 e0 = base + static_cast<u64>(q) * 256 + lane * 4;
            float v[4] = {0.f, 0.f, 0.f, 0.f};
            if (e0 < n) {
                load4<VEC>(wp, e0, n, v);
                if (LC) {
                    float l[4];
                    load4<VEC>(lp, e0, n, l);
#pragma unroll
                    for (int k = 0; k < 4; ++k) v[k] = lc_shift(v[k], l[k], a.mu);
                }
            }
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const u32 x = mag_key(v[k]);
                key[q][k] = x;
                if (e0 + k < n) {
                    above += (x > hi) ? 1u : 0u;
                    if (x - lo <= span) cmask |= 1u << (q * 4 + k);
                }
            }
        }
    }
    const u32 seg = blockIdx.x % w.n_segs;
    u32 s = above;
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) s += __shfl_down(s, d, 64);
    if (lane == 0 && s)
        atomicAdd(reinterpret_cast<unsigned long long*>(&w.seg_region[seg]), static_cast<unsigned long long>(s));   // region 0
    const u32 cnt = __popc(cmask);
    u32 incl = cnt;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const u32 o = __shfl_up(incl, d, 64);
        if (lane >= d) incl += o;
    }
    const u32 total = __shfl(incl, 63, 64);
    if (total == 0) return;
    u64 b = 0;
    if (lane == 63) b = atomicAdd(reinterpret_cast<unsigned long long*>(&w.seg_cnt[seg]), static_cast<unsigned long long>(total));
    const u32 blo = __shfl(static_cast<u32>(b), 63, 64), bhi = __shfl(static_cast<u32>(b >> 32), 63, 64);
    if (cmask == 0) return;
    u64 pos = ((static_cast<u64>(bhi) << 32) | blo) + incl - cnt;
    const u64 first = static_cast<u64>(seg) * w.seg_cap;
#pragma unroll
    for (int q = 0; q < QUADS; ++q) {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            if (cmask & (1u << (q * 4 + k))) {
                if (pos < w.seg_cap) {
                    w.cand_key[first + pos] = key[q][k];
                    w.cand_idx[first + pos] = td.flat_start + base + static_cast<u64>(q) * 256 + lane * 4 + k;
                }
                ++pos;
            }
        }
    }
}

// After the sweep: rank to find inside each window, or failure (window missed / list overflowed).
__global__ __launch_bounds__(kBlock) void k_window_check(DataArgs a, WindowArgs w) {
    __shared__ u64 s_wave[kBlock / 64];
    __shared__ u64 s_region[kMaxJ + 1];
    __shared__ SortedWindows s_win;
    __shared__ u32 s_overflow;
    const int tid = threadIdx.x;
    if (tid == 0) { s_overflow = 0; sort_windows(a.slots, w.wslots, a.J, &s_win); }
    __syncthreads();
    // every thread sums a strided share of the segments, then the workgroup adds the shares up
    u64 cnt_sum = 0;
    bool over = false;
    for (u32 seg = tid; seg < w.n_segs; seg += kBlock) {
        const u64 cnt = w.seg_cnt[seg];
        over = over || (cnt > w.seg_cap);
        cnt_sum += cnt;
    }
    if (over) s_overflow = 1;
    u64 total;
    block_excl_scan_u64(cnt_sum, s_wave, &total);
    if (tid == 0) a.ctl->cand_count = total;
    const int n = static_cast<int>(s_win.n);
    for (int r = 0; r < n; ++r) {                        // region n (below every window) is not needed
        u64 part = 0;
        // one density: the upper halves belong to the one-sweep kernel's count of non-zero codes
        for (u32 seg = tid; seg < w.n_segs; seg += kBlock) {
            const u64 v = w.seg_region[static_cast<u64>(r) * kSegs + seg];
            part += (a.J == 1) ? (v & 0xFFFFFFFFull) : v;
        }
        u64 sum;
        block_excl_scan_u64(part, s_wave, &sum);
        if (tid == 0) s_region[r] = sum;
    }
    __syncthreads();
    if (tid >= n) return;
    // keys above the window at sorted position p: regions 0..p
    u64 above = 0;
    for (int r = 0; r <= tid; ++r) above += s_region[r];
    const u32 j = s_win.slot[tid];
    Slot& s = a.slots[j];
    a.ctl->above[j] = above;
    if (s_overflow || above >= s.k) {
        s.state = kFailed;
        atomicOr(&a.ctl->window_failed, 1u);
        return;
    }
    s.remaining = s.k - above;
    const u32 hi = static_cast<u32>(w.wslots[2 * j].prefix);
    const u32 lo = static_cast<u32>(w.wslots[2 * j + 1].prefix);
    s.hi = hi;
    s.lo = lo;
    // leading digits shared by lo and hi are shared by every candidate: those levels need no counting
    u32 begin = 0;
    u64 prefix = 0;
    const int nl = n_levels(31);
    for (int level = 0; level < nl - 1; ++level) {
        const Level L = level_of(31, level);
        if (((lo ^ hi) >> L.shift) != 0) break;
        prefix = static_cast<u64>(lo >> L.shift) << L.shift;
        begin = level + 1;
    }
    s.prefix = prefix;
    s.level_begin = begin;
}

// Index rankings for the rankings whose ties are only partly kept.
__global__ __launch_bounds__(kBlock) void k_window_tie_setup(DataArgs a, WindowArgs w) {
    const int j = threadIdx.x;
    if (j >= a.J) return;
    const Slot& s = a.slots[j];
    Slot r{};
    r.state = kInactive;
    if (s.state == kDone && s.need_tie) {
        r.state = kSelecting;
        r.remaining = s.remaining;                       // the r-th lowest index = r-th largest N-1-idx
        r.k = s.remaining;
        r.n = s.n_tie;
        r.lo = r.hi = static_cast<u32>(s.prefix);        // only candidates equal to the threshold
    }
    w.wslots[j] = r;
}

// Takes over the index rankings, and re-arms the rankings that must fall back to the radix levels.
__global__ __launch_bounds__(kBlock) void k_window_finish(DataArgs a, WindowArgs w) {
    const int j = threadIdx.x;
    if (j >= a.J) return;
    Slot& s = a.slots[j];
    if (s.state == kDone && s.need_tie) {
        const Slot& r = w.wslots[j];
        if (r.state == kDone) {
            s.tie_end = a.N - r.prefix;                  // 1 + (N - 1 - ranked key)
            s.need_tie = 0;
        } else {
            s.state = kFailed;
            atomicOr(&a.ctl->window_failed, 1u);
        }
    }
    if (s.state == kFailed) {
        s.prefix = 0;
        s.remaining = s.k;
        s.n_tie = 0;
        s.tie_end = s.n;
        s.need_tie = 0;
        s.lo = s.hi = 0;
        s.level_begin = 0;
        s.path = 3;
        s.state = kSelecting;
    }
}

// ---- one density: the same steps with the level searches folded into the kernels that follow -----------

static inline int bits_for(u64 max_value) {
    int b = 1;
    while (b < 63 && (max_value >> b) != 0) ++b;
    return b;
}

// After the two levels of the sample ranking (one wavefront per boundary ranking): the boundary keys, rounded
// outwards over the low bits that two levels leave undecided.  A third level over the sample would narrow a
// window of 2^15..2^17 keys by at most 2^10 at either end.
__global__ __launch_bounds__(kBlock) void k_window_bounds(ArrayArgs ar) {
    const int j = threadIdx.x >> 6;
    if (j >= ar.n_slots) return;
    Slot& s = ar.slots[j];
    const u64* prev = array_hist(ar, 1, j);
    const SlotStep e = wave_enter_level(s, 2, 31, prev, coarse_of(ar.hist_base, ar.coarse, prev));
    if ((threadIdx.x & 63) != 0) return;
    const u32 low = (1u << level_of(31, 1).shift) - 1u;
    u32 key = s.rank_rule == kRankHi ? 0x7FFFFFFFu : 0u;                 // no bound
    if (e.state == kSelecting) {
        const u32 p = static_cast<u32>(e.prefix);
        key = s.rank_rule == kRankHi ? (p | low) : s.rank_rule == kRankLo ? p : (p | ((low + 1u) >> 1));
    } else if (e.state == kDone) {
        key = static_cast<u32>(e.prefix);
    }
    s.prefix = key;
    s.state = kDone;
}

// One density: flat indices of the candidates equal to the threshold, for the index search among ties; one
// reservation per wavefront, and the count keeps running past the capacity so that an incomplete list is
// recognised.  The threshold comes out of the last level's histogram, which every workgroup folds in itself.
__global__ __launch_bounds__(kBlock) void k_window_ties(DataArgs a, WindowArgs w, ArrayArgs ar) {
    __shared__ SlotStep s_e;
    if (threadIdx.x < 64) {
        const u64* prev = array_hist(ar, n_levels(31) - 1, 0);
        const SlotStep e = wave_enter_level(a.slots[0], n_levels(31), 31, prev, coarse_of(ar.hist_base, ar.coarse, prev));
        if (threadIdx.x == 0) s_e = e;
    }
    __syncthreads();
    if (!(s_e.state == kDone && s_e.need_tie)) return;
    const u32 T = static_cast<u32>(s_e.prefix);
    const int lane = threadIdx.x & 63;
    for (u32 seg = blockIdx.x; seg < w.n_segs; seg += gridDim.x) {
        u64 cnt = w.seg_cnt[seg];
        if (cnt > w.seg_cap) cnt = w.seg_cap;
        const u64 first = static_cast<u64>(seg) * w.seg_cap;
        const u64 rounds = (cnt + kBlock - 1) / kBlock;    // uniform over the workgroup
        for (u64 r = 0; r < rounds; ++r) {
            const u64 i = r * kBlock + threadIdx.x;
            const bool hit = (i < cnt) && w.cand_key[first + i] == T;
            const u64 ballot = __ballot(hit);
            if (ballot == 0) continue;                     // uniform over the wavefront
            const u32 n_hit = static_cast<u32>(__popcll(ballot));
            const int leader = __ffsll(static_cast<long long>(ballot)) - 1;
            u64 b = 0;
            if (lane == leader) b = atomicAdd(reinterpret_cast<unsigned long long*>(&a.ctl->tie_count), static_cast<unsigned long long>(n_hit));
            const u32 blo = __shfl(static_cast<u32>(b), leader, 64), bhi = __shfl(static_cast<u32>(b >> 32), leader, 64);
            if (hit) {
                const u64 pos = ((static_cast<u64>(bhi) << 32) | blo) + __popcll(ballot & ((static_cast<u64>(1) << lane) - 1));
                if (pos < w.tie_cap) w.tie_list[pos] = cand_flat(w.cand_idx[first + i]);
            }
        }
    }
}

// One density, one workgroup: makes the outcome of the candidate ranking the ranking's stored state.  When
// only part of the ties is kept, the r-th lowest flat index among them is found here, by radix levels on the
// index over the short tie list (lowest first).  A window that missed, a candidate list that overflowed or a
// tie list that does not hold every tie re-arms the ranking for the radix levels over the weights.
constexpr int kFinishThreads = 1024;
__global__ __launch_bounds__(kFinishThreads) void k_window_finish1(DataArgs a, WindowArgs w, ArrayArgs ar, int idx_bits) {
    __shared__ SlotStep s_e;
    __shared__ __align__(8) u32 s_hist[kBins];
    __shared__ u64 s_pick[2];              // chosen bin, rank inside it
    const int tid = threadIdx.x;
    Slot& s = a.slots[0];
    const u32 state0 = s.state;
    if (state0 != kSelecting && state0 != kFailed) return;               // k == 0: nothing was ranked
    if (tid < 64) {
        const u64* prev = array_hist(ar, n_levels(31) - 1, 0);
        const SlotStep e = wave_enter_level(s, n_levels(31), 31, prev, coarse_of(ar.hist_base, ar.coarse, prev));
        if (tid == 0) s_e = e;
    }
    __syncthreads();
    const SlotStep e = s_e;
    bool ok = (e.state == kDone);
    u64 tie_end = s.n;
    if (ok && e.need_tie) {
        const u64 n_t = a.ctl->tie_count;
        if (n_t != e.n_tie || n_t > w.tie_cap) {
            ok = false;                                                  // the list does not hold every tie
        } else if (n_t <= static_cast<u64>(kFinishThreads)) {
            // the usual case, a handful of ties: one index per thread, ranked by counting the lower ones
            u64* s_idx = reinterpret_cast<u64*>(s_hist);                 // kBins words hold kFinishThreads indices
            const u64 mine = (static_cast<u64>(tid) < n_t) ? w.tie_list[tid] : ~static_cast<u64>(0);
            s_idx[tid] = mine;
            if (tid == 0) s_pick[0] = s.n - 1;
            __syncthreads();
            if (static_cast<u64>(tid) < n_t) {
                u64 lower = 0;
                for (u64 i = 0; i < n_t; ++i) lower += (s_idx[i] < mine) ? 1u : 0u;
                if (lower + 1 == e.remaining) s_pick[0] = mine;          // flat indices are distinct: one thread
            }
            __syncthreads();
            tie_end = s_pick[0] + 1;
        } else {
            u64 prefix = 0, r = e.remaining;
            for (int level = 0; level < n_levels(idx_bits); ++level) {   // uniform
                const Level lv = level_of(idx_bits, level);
                const int nb = 1 << lv.bits;
                for (int i = tid; i < nb; i += kFinishThreads) s_hist[i] = 0;
                __syncthreads();
                for (u64 i = tid; i < n_t; i += kFinishThreads) {
                    const u64 idx = w.tie_list[i];
                    if (((idx ^ prefix) >> lv.hi_shift) == 0) atomicAdd(&s_hist[static_cast<u32>(idx >> lv.shift) & (nb - 1)], 1u);
                }
                __syncthreads();
                if (tid < 64) {                                          // ascending walk: the bin that holds the r-th lowest
                    constexpr int kPerMax = kBins / 64;
                    const int per = (nb + 63) / 64;
                    u64 sum = 0;
                    u32 c[kPerMax];
#pragma unroll
                    for (int i = 0; i < kPerMax; ++i) {
                        const int bin = tid * per + i;
                        c[i] = (i < per && bin < nb) ? s_hist[bin] : 0u;
                        sum += c[i];
                    }
                    const u64 incl = wave_incl_scan_u64(sum);
                    u64 before = incl - sum;
                    if (before < r && r <= incl) {
#pragma unroll
                        for (int i = 0; i < kPerMax; ++i) {
                            if (before < r && r <= before + c[i]) { s_pick[0] = static_cast<u64>(tid * per + i); s_pick[1] = r - before; }
                            before += c[i];
                        }
                    }
                }
                __syncthreads();
                prefix |= s_pick[0] << lv.shift;
                r = s_pick[1];
                __syncthreads();
            }
            tie_end = prefix + 1;
        }
    }
    if (tid != 0) return;
    if (ok) {
        s.prefix = e.prefix;
        s.remaining = e.remaining;
        s.n_tie = e.n_tie;
        s.need_tie = 0;
        s.tie_end = tie_end;
        s.state = kDone;
    } else {
        s.prefix = 0;
        s.remaining = s.k;
        s.n_tie = 0;
        s.tie_end = s.n;
        s.need_tie = 0;
        s.lo = s.hi = 0;
        s.level_begin = 0;
        s.path = 3;
        s.state = kSelecting;
        atomicOr(&a.ctl->window_failed, 1u);
    }
}

// Workgroups of 256 threads for the candidate-segment kernels (one per 2048 entries, at most 1024).
static inline unsigned array_grid(u64 n) {
    u64 b = (n + kBlock * 8 - 1) / (kBlock * 8);
    if (b > 1024) b = 1024;     // measured: time falls with the workgroup count up to here
    if (b == 0) b = 1;
    return static_cast<unsigned>(b);
}

// Workgroups of kArrayThreads threads for k_hist_array: the same number of threads in a quarter of the
// workgroups.
static inline unsigned hist_array_grid(u64 n) {
    u64 b = (n + kArrayThreads * 8 - 1) / (kArrayThreads * 8);
    if (b > 256) b = 256;       // measured: 256 and 512 equal, 128 slower
    if (b == 0) b = 1;
    return static_cast<unsigned>(b);
}

template <bool IDX>
static condensa_status rank_array(const ArrayArgs& ar, Control* ctl, u32* tie_flag, hipStream_t st) {
    for (int level = 0; level < n_levels(ar.key_bits); ++level) {
        hipLaunchKernelGGL((k_hist_array<IDX>), dim3(hist_array_grid(ar.n_host)), dim3(kArrayThreads), 0, st, ar, level);
        CONDENSA_LAUNCH_CHECK();
        // with a shared level-0 histogram every ranking reads group 0 of `shared0` (J = n_slots)
        hipLaunchKernelGGL(k_scan_level, dim3(ar.n_slots), dim3(kBlock), 0, st, ar.slots,
                           static_cast<const u64*>(ar.shared0), ar.hist, ar.shared0 ? ar.n_slots : 1, ar.key_bits,
                           level, ctl, 0, tie_flag);
        CONDENSA_LAUNCH_CHECK();
    }
    return CONDENSA_OK;
}

// Selection and apply in one sweep (defined with its fix-up kernels in k_fused.h).
template <bool LC, bool VEC, int QUADS, bool PQ>
__global__ __launch_bounds__(64) void k_window_fused(DataArgs a, WindowArgs w);

struct FusedRequest {
    const OutDesc* out;    // device output table
    bool vec_out;          // every output pointer allows 128-bit accesses
    bool pq;               // L-C step whose theta is also rounded to binary16
    WindowArgs* w_out;     // receives the window arguments for the fix-up pass
};

// float4 per thread of the one-sweep kernel, measured on 1.2 G weights: the L-C form (2 reads, 3 writes)
// is fastest with 1 (3.96 ms; 2: 4.16, 4: 4.13), the pruning form (1 read, theta + mask) with 4
// (1.79 ms; 2: 1.91, 1: 2.37).
constexpr int kFusedQuadsLC = 1, kFusedQuadsPrune = 4;

// Window arguments shared by the two launch sequences below; *sweep_groups gets the sweep's grid.
template <bool LC>
static WindowArgs make_window_args(const DataArgs& a, const Layout& L, void* ws, const Config& cfg,
                                   const FusedRequest* fused, u64* sweep_groups) {
    char* base = static_cast<char*>(ws);
    WindowArgs w{};
    w.sample = reinterpret_cast<u32*>(base + L.sample);
    w.cand_key = reinterpret_cast<u32*>(base + L.cand_key);
    w.cand_idx = reinterpret_cast<u64*>(base + L.cand_idx);
    w.wslots = a.slots + a.J;
    const u64 quads = a.n_chunks * (kChunk / 4);
    w.n_units = L.sample_cap / kSampleUnit < quads ? L.sample_cap / kSampleUnit : quads;
    w.stride = quads / w.n_units;
    w.cand_cap = L.cand_cap;
    w.seg_cnt = reinterpret_cast<u64*>(base + L.seg);
    w.seg_region = w.seg_cnt + kSegs;
    constexpr int kWaveQuads = LC ? 4 : 8;                       // 8 KB of input per wavefront: measured best of 4, 8, 16 KB
    constexpr int kFusedQuads = LC ? kFusedQuadsLC : kFusedQuadsPrune;
    const bool fuse = fused != nullptr && a.J == 1;
    *sweep_groups = fuse ? a.n_chunks * (kChunk / (256 * kFusedQuads))
                         : (a.J == 1) ? a.n_chunks * (kChunk / (256 * kWaveQuads)) : a.n_chunks;
    w.cand_w = reinterpret_cast<float*>(base + L.cand_w);
    w.cand_lam = reinterpret_cast<float*>(base + L.cand_lam);
    w.out = fuse ? fused->out : nullptr;
    w.sorted = reinterpret_cast<SortedWindows*>(base + L.sorted_windows);
    w.n_segs = static_cast<u32>(*sweep_groups < static_cast<u64>(kSegs) ? *sweep_groups : static_cast<u64>(kSegs));
    w.seg_cap = L.cand_cap / w.n_segs;
    w.margin16 = static_cast<int>(cfg[CONDENSA_OPT_WINDOW_MARGIN]);
    w.tie_list = reinterpret_cast<u64*>(base + L.sample);        // the sample is dead once its ranking is done
    w.tie_cap = L.sample_cap / 2;
    w.hist_main = a.histx + static_cast<u64>(2 * a.J) * kBins;           // behind the radix levels' own histograms
    w.hist_aux = w.hist_main + static_cast<u64>(3 * a.J) * kBins;
    w.hist_shared0 = w.hist_aux + static_cast<u64>(2 * (2 * a.J + 1)) * kBins;
    return w;
}

// The one-sweep or selection-only sweep kernel of a single density.
template <bool LC, bool VEC>
static condensa_status launch_single_sweep(const DataArgs& a, const WindowArgs& w, const FusedRequest* fused,
                                           u64 sweep_groups, hipStream_t st) {
    constexpr int kWaveQuads = LC ? 4 : 8;
    constexpr int kFusedQuads = LC ? kFusedQuadsLC : kFusedQuadsPrune;
    const dim3 fg(static_cast<unsigned>(sweep_groups));
    if (fused && LC && fused->pq) {
        if (VEC && fused->vec_out) hipLaunchKernelGGL((k_window_fused<LC, true, kFusedQuads, LC>), fg, dim3(64), 0, st, a, w);
        else                       hipLaunchKernelGGL((k_window_fused<LC, false, kFusedQuads, LC>), fg, dim3(64), 0, st, a, w);
    } else if (fused && VEC && fused->vec_out)
        hipLaunchKernelGGL((k_window_fused<LC, true, kFusedQuads, false>), fg, dim3(64), 0, st, a, w);
    else if (fused)
        hipLaunchKernelGGL((k_window_fused<LC, false, kFusedQuads, false>), fg, dim3(64), 0, st, a, w);
    else
        hipLaunchKernelGGL((k_window_sweep_wave<LC, VEC, kWaveQuads>), fg, dim3(64), 0, st, a, w);
    CONDENSA_LAUNCH_CHECK();
    return CONDENSA_OK;
}

// One density: 10 launches where the general sequence below needs 24 or more.  The sample is ranked over two levels
// (the host has filled in the three boundary rankings; their ranks follow from the sample's size on the device),
// the candidates over the levels that their window leaves open, every level search folded into the kernel that
// follows it, and the index search among ties runs on the short tie list inside the finishing workgroup.
template <bool LC, bool VEC>
static condensa_status launch_window_path_single(const DataArgs& a, const Layout& L, void* ws, hipStream_t st,
                                                 const Config& cfg, const FusedRequest* fused) {
    if (a.n_chunks == 0) return CONDENSA_OK;
    u64 sweep_groups = 0;
    WindowArgs w = make_window_args<LC>(a, L, ws, cfg, fused, &sweep_groups);
    condensa_status rc;
    {
        PhaseTimer timer(CONDENSA_PHASE_SAMPLE, st, cfg);
        ArrayArgs ar{};
        ar.keys = w.sample; ar.n_host = w.n_units * kSampleUnit; ar.slots = w.wslots; ar.n_slots = 3;
        ar.hist = w.hist_aux; ar.key_bits = 31; ar.shared0 = w.hist_shared0; ar.merged = 1;
        ar.hist_base = a.hist0; ar.coarse = a.coarse;
        u64 sample_groups = (w.n_units + kSampleHistThreads - 1) / kSampleHistThreads;
        if (sample_groups > 512) sample_groups = 512;
        hipLaunchKernelGGL((k_sample_hist<LC, VEC>), dim3(static_cast<unsigned>(sample_groups)), dim3(kSampleHistThreads), 0, st, a, w, ar);
        CONDENSA_LAUNCH_CHECK();
        hipLaunchKernelGGL((k_hist_array<false>), dim3(hist_array_grid(ar.n_host)), dim3(kArrayThreads), 0, st, ar, 1);
        CONDENSA_LAUNCH_CHECK();
        hipLaunchKernelGGL(k_window_bounds, dim3(1), dim3(kBlock), 0, st, ar);
        CONDENSA_LAUNCH_CHECK();
    }
    {
        PhaseTimer timer(CONDENSA_PHASE_SWEEP, st, cfg);
        rc = launch_single_sweep<LC, VEC>(a, w, fused, sweep_groups, st);
        if (rc != CONDENSA_OK) return rc;
    }
    PhaseTimer timer(CONDENSA_PHASE_RESOLVE, st, cfg);
    hipLaunchKernelGGL(k_window_check, dim3(1), dim3(kBlock), 0, st, a, w);
    CONDENSA_LAUNCH_CHECK();
    ArrayArgs cr{};
    cr.keys = w.cand_key; cr.seg_cnt = w.seg_cnt; cr.seg_cap = w.seg_cap; cr.n_segs = w.n_segs;
    cr.n_host = static_cast<u64>(w.n_segs) * kBlock * 8; cr.slots = a.slots; cr.n_slots = 1;
    cr.hist = w.hist_main; cr.key_bits = 31; cr.merged = 1; cr.hist_base = a.hist0; cr.coarse = a.coarse;
    for (int level = 0; level < n_levels(31); ++level) {
        hipLaunchKernelGGL((k_hist_array<false>), dim3(hist_array_grid(cr.n_host)), dim3(kArrayThreads), 0, st, cr, level);
        CONDENSA_LAUNCH_CHECK();
    }
    hipLaunchKernelGGL(k_window_ties, dim3(array_grid(cr.n_host)), dim3(kBlock), 0, st, a, w, cr);
    CONDENSA_LAUNCH_CHECK();
    hipLaunchKernelGGL(k_window_finish1, dim3(1), dim3(kFinishThreads), 0, st, a, w, cr, bits_for(a.N - 1));
    CONDENSA_LAUNCH_CHECK();
    if (fused && fused->w_out) *fused->w_out = w;
    return CONDENSA_OK;
}

// Any number of densities: every level search is a launch of its own (k_scan_level), the boundary ranks come
// from k_window_ranks, and the index search among ties ranks the candidate list itself.
template <bool LC, bool VEC>
static condensa_status launch_window_path(const DataArgs& a, const Layout& L, void* ws, hipStream_t st,
                                          const Config& cfg) {
    if (a.n_chunks == 0) return CONDENSA_OK;
    u64 sweep_groups = 0;
    WindowArgs w = make_window_args<LC>(a, L, ws, cfg, nullptr, &sweep_groups);
    u64* hist_main = w.hist_main;                                // [J]
    u64* hist_aux = w.hist_aux;                                  // [2J]
    condensa_status rc;
    {
        PhaseTimer timer(CONDENSA_PHASE_SAMPLE, st, cfg);
        hipLaunchKernelGGL((k_sample<LC, VEC>), dim3(static_cast<unsigned>((w.n_units + kBlock - 1) / kBlock)), dim3(kBlock), 0, st, a, w);
        CONDENSA_LAUNCH_CHECK();
        hipLaunchKernelGGL(k_window_ranks, dim3(1), dim3(kBlock), 0, st, a, w);
        CONDENSA_LAUNCH_CHECK();
        ArrayArgs ar{};
        ar.keys = w.sample; ar.n_host = w.n_units * kSampleUnit; ar.slots = w.wslots; ar.n_slots = 2 * a.J;
        ar.hist = hist_aux; ar.key_bits = 31;
        ar.shared0 = w.hist_shared0;                                  // boundary rankings share level 0
        rc = rank_array<false>(ar, a.ctl, &a.ctl->unused_flag, st);
        if (rc != CONDENSA_OK) return rc;
    }
    {
        PhaseTimer timer(CONDENSA_PHASE_SWEEP, st, cfg);
        hipLaunchKernelGGL(k_window_sort, dim3(1), dim3(64), 0, st, a, w);
        CONDENSA_LAUNCH_CHECK();
        hipLaunchKernelGGL((k_window_sweep<LC, VEC>), dim3(static_cast<unsigned>(sweep_groups)), dim3(kBlock), 0, st, a, w);
        CONDENSA_LAUNCH_CHECK();
    }
    PhaseTimer timer(CONDENSA_PHASE_RESOLVE, st, cfg);
    hipLaunchKernelGGL(k_window_check, dim3(1), dim3(kBlock), 0, st, a, w);
    CONDENSA_LAUNCH_CHECK();
    {
        ArrayArgs ar{};
        ar.keys = w.cand_key; ar.seg_cnt = w.seg_cnt; ar.seg_cap = w.seg_cap; ar.n_segs = w.n_segs;
        ar.n_host = static_cast<u64>(w.n_segs) * kBlock * 8; ar.slots = a.slots; ar.n_slots = a.J;
        ar.hist = hist_main; ar.key_bits = 31;
        rc = rank_array<false>(ar, a.ctl, &a.ctl->need_tie_w, st);
        if (rc != CONDENSA_OK) return rc;
    }
    hipLaunchKernelGGL(k_window_tie_setup, dim3(1), dim3(kBlock), 0, st, a, w);
    CONDENSA_LAUNCH_CHECK();
    {
        ArrayArgs ar{};
        ar.keys = w.cand_key; ar.idx = w.cand_idx; ar.seg_cnt = w.seg_cnt; ar.seg_cap = w.seg_cap; ar.n_segs = w.n_segs;
        ar.n_host = static_cast<u64>(w.n_segs) * kBlock * 8; ar.N = a.N;
        ar.slots = w.wslots; ar.n_slots = a.J; ar.hist = hist_aux; ar.key_bits = bits_for(a.N - 1);
        ar.gate = &a.ctl->need_tie_w;
        rc = rank_array<true>(ar, a.ctl, &a.ctl->unused_flag, st);
        if (rc != CONDENSA_OK) return rc;
    }
    hipLaunchKernelGGL(k_window_finish, dim3(1), dim3(kBlock), 0, st, a, w);
    CONDENSA_LAUNCH_CHECK();
    return CONDENSA_OK;
}

}  // namespace condensa
