// Exact k-th-largest selection by most-significant-digit radix levels with workgroup-private LDS
// histograms, and the deterministic tie rule (lowest index first).
// Section 3.1: the magnitude threshold that realises a given sparsity; Section 3.3: the C step.
#pragma once
#include "common.h"

namespace condensa {

// Small block of device-side flags and counters, zeroed at the start of every call.
struct Control {
    u32 need_tie;          // radix path: some ranking needs the index search among ties
    u32 window_failed;     // some ranking of the window path must fall back to the radix levels
    u32 need_tie_w;        // window path: some ranking needs the index search among candidates
    u32 unused_flag;       // sink for rankings whose tie state does not matter
    u64 cand_count;        // candidates written by the window sweep (may exceed the capacity)
    u64 sample_count;      // valid sample elements
    u64 above[kMaxJ];      // window sweep: keys above each window's upper bound
    u64 tie_count;         // candidates equal to the threshold (the tie list holds the first tie_cap)
    u64 nnz_delta;         // prune + binary16 L-C step: what the fix-up pass changes about the one-sweep kernel's
                           // count of non-zero codes (two's complement)
    u64 pad[2];
};
static_assert(sizeof(Control) == 32 + 8 * kMaxJ + 32, "Control layout");

struct DataArgs {
    const TensorDesc* td;
    Slot* slots;
    u64* hist0;            // [n_groups][kBins]   first level, shared by the densities of a group
    u64* histx;            // [n_slots][kBins]    later levels
    u32* tiecnt;           // [J][n_chunks]
    Control* ctl;
    const u32* chunk_map;  // [n_chunks] tensor that owns each chunk
    u64 n_chunks;
    u64 N;                 // total elements of the call
    int n_tensors;
    int J;                 // rankings (densities) per group
    int per_tensor;        // 1: group = tensor, 0: one group
    int only_failed;       // 1: runs as the fallback of the window path (skip when nothing failed)
    int streaming;         // 1: the inputs exceed the caches, so repeated sweeps gain nothing from keeping lines
    float mu;
    int merged;            // 1 (GLOBAL scope): every level kernel folds in the previous level's histogram itself
                           // (wave_enter_level), one histogram per ranking and level; 0: k_scan_level runs between levels
    u64* coarse;           // merged form: kCoarse sums per histogram, in the order of the histograms from hist0 on
    u64* nnz_seg;          // prune + binary16 L-C step: non-zero codes written by the apply sweep, per counter segment (or NULL)
    u32* tiehit;           // [n_chunks] set by the last radix level where a chunk holds a key that agrees with some
                           // ranking on all earlier digits: only those chunks can hold ties of a threshold
    // Merged form: the last radix level also lists (key, flat index) of the keys that agree with ranking j on
    // all earlier digits - a thousand of 20 M weights - so that the ties of the threshold are usually found
    // in that list, without another sweep over the weights (NULL: no lists).
    u64* tl_cnt;           // [kMaxJ] entries offered per ranking; above kTieListCap: the list is incomplete
    u32* tl_key;           // [J][kTieListCap]
    u64* tl_idx;           // [J][kTieListCap]
    u64 small_cap;         // > 0: a small call (k_small.h) - tl_key / tl_idx hold this many entries as ONE list of the
                           // keys that share their leading digit with a threshold, counted by tl_cnt[0]
};
constexpr u32 kTieListCap = 4096;      // entries per ranking's list
constexpr u32 kTieListGroup = 128;     // entries one workgroup may offer to the lists.  It buffers them in LDS and reserves
                                       // room with one atomic per ranking at its end (an atomic per entry would queue a
                                       // thousand of them on one address: +13 us on the 20 M-weight call); a workgroup
                                       // that finds more declares every list incomplete, and the sweep over the weights
                                       // counts the ties as before
constexpr u32 kTieListTies = 512;      // ties of one threshold resolved from the list (ranked in LDS by one workgroup)

// The tie search of ranking j can use its list: every key of the last level's bins is in it, and the ties fit.
__device__ inline bool tie_list_usable(const DataArgs& a, int j, u64 n_tie) {
    return a.tl_cnt != nullptr && a.tl_cnt[j] <= kTieListCap && n_tie <= kTieListTies;
}
constexpr int kNnzSegs = 1024;   // counter segments of the apply sweeps (one address would serialise ~10^6 atomics)

// Every histogram of the merged form comes with kCoarse sums over runs of consecutive bins, so that the
// workgroups that fold a level in read ~100 counters instead of 2048 (hundreds of workgroups walking the same
// 16 KB at once queue up on a few cache channels).
constexpr int kCoarse = 64;
__device__ inline int coarse_run(int nb) { return (nb + kCoarse - 1) / kCoarse; }    // bins per coarse sum
__device__ inline u64* coarse_of(u64* hist_base, u64* coarse_base, const u64* fine) {
    return coarse_base + static_cast<u64>(fine - hist_base) / kBins * kCoarse;
}

// Histogram of radix level `level` (>= 1) of ranking s over the weights; level 0 is shared per group (hist0).
__device__ inline u64* data_hist(const DataArgs& a, int level, u64 s) {
    return a.histx + (a.merged ? static_cast<u64>(level - 1) * static_cast<u64>(a.J) + s : s) * kBins;
}

// ---- wavefront / workgroup scans ---------------------------------------------------------------

__device__ inline u64 shfl_up_u64(u64 v, int d) {
    const u32 lo = __shfl_up(static_cast<u32>(v), d, 64);
    const u32 hi = __shfl_up(static_cast<u32>(v >> 32), d, 64);
    return (static_cast<u64>(hi) << 32) | lo;
}

__device__ inline u64 wave_incl_scan_u64(u64 v) {
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const u64 o = shfl_up_u64(v, d);
        if (lane >= d) v += o;
    }
    return v;
}

// Exclusive scan over the 256 threads of a workgroup in thread order; *total gets the sum.
// s_wave must hold kBlock / 64 entries.  All threads must call it.
__device__ inline u64 block_excl_scan_u64(u64 v, u64* s_wave, u64* total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const u64 incl = wave_incl_scan_u64(v);
    __syncthreads();                       // s_wave may still be read from a previous call
    if (lane == 63) s_wave[wave] = incl;
    __syncthreads();
    u64 before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < kBlock / 64; ++w) {
        const u64 t = s_wave[w];
        if (w < wave) before += t;
        all += t;
    }
    *total = all;
    return before + incl - v;
}

__device__ inline SlotStep slot_canonical(const Slot& s) {
    SlotStep e;
    e.prefix = s.prefix; e.remaining = s.remaining; e.n_tie = s.n_tie; e.state = s.state; e.need_tie = s.need_tie;
    return e;
}

// Rank of a boundary ranking on a sample of S keys.  The number of sample keys above the true threshold is
// (close to) binomial; sample units of 4 neighbours may be correlated, so the standard deviation is taken as
// if every unit were one draw.  A bound that falls outside the sample ends the ranking at once: no upper
// bound (prefix = largest key) or no lower bound (prefix = 0).
__device__ inline void sample_rank(const Slot& s, u64 S, SlotStep* e) {
    const double p = s.p;
    const double ks = p * static_cast<double>(S);
    const double sd = sqrt(4.0 * static_cast<double>(S) * p * (1.0 - p));
    const double m = static_cast<double>(s.margin16) / 16.0 * sd + 2.0;
    double r;
    if (s.rank_rule == kRankHi) {
        r = floor(ks - m);
        if (S == 0 || r < 1.0) { e->state = kDone; e->prefix = 0x7FFFFFFFu; return; }
    } else if (s.rank_rule == kRankLo) {
        r = ceil(ks + m) + 1.0;
        if (S == 0 || r > static_cast<double>(S)) { e->state = kDone; e->prefix = 0; return; }
    } else {
        r = floor(ks + 0.5);
        if (S == 0) { e->state = kDone; e->prefix = 0; return; }
        if (r < 1.0) r = 1.0;
        if (r > static_cast<double>(S)) r = static_cast<double>(S);
    }
    e->remaining = static_cast<u64>(r);
}

// State of ranking `s` on entering radix level L: the stored state of level L - 1 with the histogram of that
// level (`hist_prev` and its coarse sums, complete: an earlier kernel filled them) folded in.  Bins are walked
// from the top; the bin b with  #(keys in higher bins) < remaining <= #(keys in bins >= b)  extends the prefix.
// After the last level the prefix is the threshold key, `remaining` the number of ties to keep and n_tie the
// number of keys equal to the threshold.  Called by all 64 lanes of a wavefront; every lane returns the same value.
__device__ inline SlotStep wave_enter_level(const Slot& s, int L, int key_bits, const u64* __restrict__ hist_prev,
                                            const u64* __restrict__ coarse_prev) {
    SlotStep cur = slot_canonical(s);
    const int b = static_cast<int>(s.level_begin);
    if (cur.state != kSelecting || L <= b) return cur;          // no level search under way, or level not reached yet
    if (L - 1 > b) cur = s.step[(L - 1) & 1];
    if (cur.state != kSelecting) return cur;                     // failed at an earlier level
    const Level lv = level_of(key_bits, L - 1);
    const int nb = 1 << lv.bits;
    const int run = coarse_run(nb);
    const int lane = threadIdx.x & 63;
    // coarse sums, highest bins first: lane l takes run kCoarse - 1 - l
    const int crun = kCoarse - 1 - lane;
    const u64 csum = (crun * run < nb) ? coarse_prev[crun] : 0;
    const u64 cincl = wave_incl_scan_u64(csum);
    const u64 total = (static_cast<u64>(__shfl(static_cast<u32>(cincl >> 32), 63, 64)) << 32) | __shfl(static_cast<u32>(cincl), 63, 64);
    if (s.rank_rule != kRankGiven && L - 1 == b) {
        sample_rank(s, total, &cur);
        if (cur.state != kSelecting) return cur;
    }
    const u64 r = cur.remaining;
    if (total < r) {                                             // the wanted rank is not in this population
        cur.state = kFailed;
        return cur;
    }
    const bool mine = (cincl - csum) < r && r <= cincl;          // exactly one lane
    const int src = __ffsll(static_cast<long long>(__ballot(mine))) - 1;
    const int run_found = kCoarse - 1 - src;
    u64 before = cincl - csum;
    before = (static_cast<u64>(__shfl(static_cast<u32>(before >> 32), src, 64)) << 32) | __shfl(static_cast<u32>(before), src, 64);
    // the bins of that run, highest first: lane l takes bin (run_found + 1) * run - 1 - l
    const int bin = (run_found + 1) * run - 1 - lane;
    const u64 f = (lane < run && bin < nb) ? hist_prev[bin] : 0;
    const u64 fincl = wave_incl_scan_u64(f);
    const bool mine2 = before + (fincl - f) < r && r <= before + fincl;
    const int src2 = __ffsll(static_cast<long long>(__ballot(mine2))) - 1;
    const u64 rem_l = r - (before + (fincl - f));
    const u64 rem = (static_cast<u64>(__shfl(static_cast<u32>(rem_l >> 32), src2, 64)) << 32) | __shfl(static_cast<u32>(rem_l), src2, 64);
    const u64 cnt = (static_cast<u64>(__shfl(static_cast<u32>(f >> 32), src2, 64)) << 32) | __shfl(static_cast<u32>(f), src2, 64);
    const u32 bin_found = static_cast<u32>((run_found + 1) * run - 1 - src2);
    cur.prefix |= static_cast<u64>(bin_found) << lv.shift;
    cur.remaining = rem;
    cur.n_tie = cnt;
    if (L - 1 == n_levels(key_bits) - 1) {
        cur.state = kDone;
        cur.need_tie = rem < cnt ? 1u : 0u;
    }
    return cur;
}

// First kernel of every call: clears the flag / counter / histogram region and writes the
// chunk -> tensor map (a kernel rather than a memset: memset nodes do not belong in work that a caller may
// capture in a graph, as the caller of the allocation-free entry point may).
__global__ __launch_bounds__(kBlock) void k_prepare(u64* zero, u64 n_words, const TensorDesc* td, int n_tensors,
                                                    u32* chunk_map, u64 n_chunks) {
    const u64 stride = static_cast<u64>(gridDim.x) * kBlock;
    const u64 i0 = static_cast<u64>(blockIdx.x) * kBlock + threadIdx.x;
    for (u64 i = i0; i < n_words; i += stride) zero[i] = 0;
    for (u64 c = i0; c < n_chunks; c += stride) chunk_map[c] = static_cast<u32>(tensor_of_chunk(td, n_tensors, c));
}

// ---- histogram of one radix level over the weights ----------------------------------------------
//
// Every workgroup sweeps a contiguous range of chunks and keeps its counts in LDS; they are added
// to the global histogram when the group (tensor under PER_TENSOR scope) changes and at the end.
// Level 0 has no prefix to match, so the densities of a group share one histogram; later levels
// keep one histogram per ranking, kSlotBatch rankings per sweep of the range.  At those levels a table
// over the leading digit says which rankings of the batch a key can belong to (a bit per ranking), so
// a key costs one LDS read unless it shares its leading digit with a threshold.

// Rankings of a batch whose prefix starts with each leading digit; built by one thread (<= 14 entries).
__device__ inline void build_digit_table(u16* tab, const u32* prefix, const u32* active, int nj, int tid) {
    const Level L0 = level_of(31, 0);
    for (int i = tid; i < kBins; i += kBlock) tab[i] = 0;
    __syncthreads();
    if (tid == 0)
        for (int j = 0; j < nj; ++j)
            if (active[j]) tab[prefix[j] >> L0.shift] |= static_cast<u16>(1u << j);
}

// The workgroup is 1024 threads under GLOBAL scope (few, wide workgroups: fewer flushes of the LDS
// histograms through global atomics, and enough wavefronts per compute unit even when J histograms of
// 4 KB each limit the workgroups per unit), 256 under PER_TENSOR scope, where the histograms change with
// the tensor.  Each quarter of a wide workgroup takes a chunk of its own.
template <bool LC, bool VEC>
__global__ __launch_bounds__(1024) void k_hist_data(DataArgs a, int level, u64 chunks_per_block) {
    extern __shared__ u32 s_hist[];       // level 0: kBins words; later levels: min(J, kSlotBatch) x 1024 words
    __shared__ u16 s_tab[kBins];
    __shared__ u32 s_prefix[kSlotBatch];
    __shared__ u32 s_active[kSlotBatch];
    __shared__ u32 s_mprefix[kMaxJ];      // merged form: the rankings' state on entering this level
    __shared__ u32 s_mactive[kMaxJ];
    __shared__ u32 s_ln;                  // last level: entries this workgroup found for the rankings' lists
    __shared__ u32 s_lkey[kTieListGroup];
    __shared__ u64 s_lidx[kTieListGroup];
    __shared__ u32 s_lj[kTieListGroup];
    __shared__ u64 s_lbase[kMaxJ];
    __shared__ u32 s_any;

    if (a.only_failed && a.ctl->window_failed == 0) return;
    if (threadIdx.x == 0) s_ln = 0;       // ordered before its use by the barriers below
    if (a.merged && level > 0) {          // one group; every workgroup derives the same state, workgroup 0 stores it
        const int n_waves = static_cast<int>(blockDim.x) >> 6;
        for (int j = static_cast<int>(threadIdx.x) >> 6; j < a.J; j += n_waves) {
            const u64* prev = level == 1 ? a.hist0 : data_hist(a, level - 1, j);
            const SlotStep e = wave_enter_level(a.slots[j], level, 31, prev, coarse_of(a.hist0, a.coarse, prev));
            if ((threadIdx.x & 63) == 0) {
                s_mprefix[j] = static_cast<u32>(e.prefix);
                s_mactive[j] = (e.state == kSelecting) ? 1u : 0u;
                if (blockIdx.x == 0) a.slots[j].step[level & 1] = e;
            }
        }
        __syncthreads();
    }
    const u64 c0 = static_cast<u64>(blockIdx.x) * chunks_per_block;
    if (c0 >= a.n_chunks) return;
    const u64 c1 = (c0 + chunks_per_block < a.n_chunks) ? c0 + chunks_per_block : a.n_chunks;

    const Level L = level_of(31, level);
    const Level L0 = level_of(31, 0);
    const int nb = 1 << L.bits;
    const int wide = static_cast<int>(blockDim.x);
    const int n_sub = wide / kBlock;                      // quarters (1 in a 256-thread workgroup)
    const int sub = static_cast<int>(threadIdx.x) / kBlock;
    const int tid = static_cast<int>(threadIdx.x) % kBlock;
    const int wtid = static_cast<int>(threadIdx.x);
    const int n_batches = (level == 0) ? 1 : (a.J + kSlotBatch - 1) / kSlotBatch;

    u32 p0 = 0;                                           // the prefix when a batch holds a single ranking
    bool single = false;
    // Last level: a chunk that holds a key matching a ranking's earlier digits is flagged (plain stores of 1:
    // whoever writes, writes the same), so that the tie search reads those chunks only.
    const bool last = (level == n_levels(31) - 1) && level > 0;
    u32* hit = nullptr;
    const bool listing = last && a.merged && a.tl_cnt != nullptr;
    int list_j0 = 0;                                      // first ranking of the batch being counted
    u64 chunk_flat = 0;                                   // flat index of the current chunk's first element
    // last level: the key (element `off` of the current chunk) agrees with ranking j on every earlier digit
    auto list_key = [&](int j, u32 key, u32 off) {
        *hit = 1u;
        if (!listing) return;
        const u32 mine = atomicAdd(&s_ln, 1u);
        if (mine < kTieListGroup) {
            s_lkey[mine] = key;
            s_lidx[mine] = chunk_flat + off;
            s_lj[mine] = static_cast<u32>(j);
        }
    };
    auto count_key = [&](u32 key, u32 off) {
        if (level == 0) {
            atomicAdd(&s_hist[key >> L.shift], 1u);
        } else if (single) {                              // one ranking: compare with its prefix, no table look-up
            if (((key ^ p0) >> L.hi_shift) == 0) {
                atomicAdd(&s_hist[(key >> L.shift) & (nb - 1)], 1u);
                if (last) list_key(list_j0, key, off);
            }
        } else {
            u32 m = s_tab[key >> L0.shift];
            const u32 digit = (key >> L.shift) & (nb - 1);
            while (m) {
                const int j = __ffs(m) - 1;
                m &= m - 1;
                if (((key ^ s_prefix[j]) >> L.hi_shift) == 0) {
                    atomicAdd(&s_hist[j * nb + digit], 1u);
                    if (last) list_key(list_j0 + j, key, off);
                }
            }
        }
    };
    auto flush = [&](long long group, int j0, int n_hist) {
        for (int i = wtid; i < n_hist * nb; i += wide) {
            const u32 v = s_hist[i];
            if (v) {
                u64* dst = (level == 0) ? a.hist0 + static_cast<u64>(group) * kBins + i
                                        : data_hist(a, level, static_cast<u64>(group) * a.J + j0 + i / nb) + (i % nb);
                atomicAdd(reinterpret_cast<unsigned long long*>(dst), static_cast<unsigned long long>(v));
            }
        }
        if (a.merged) {                                    // the coarse sums of the same counts
            const int run = coarse_run(nb);
            for (int i = wtid; i < n_hist * kCoarse; i += wide) {
                const int h = i / kCoarse, c = i % kCoarse;
                u32 v = 0;
                for (int t = c * run; t < (c + 1) * run && t < nb; ++t) v += s_hist[h * nb + t];
                if (v) {
                    u64* fine = (level == 0) ? a.hist0 + static_cast<u64>(group) * kBins
                                             : data_hist(a, level, static_cast<u64>(group) * a.J + j0 + h);
                    atomicAdd(reinterpret_cast<unsigned long long*>(coarse_of(a.hist0, a.coarse, fine) + c), static_cast<unsigned long long>(v));
                }
            }
        }
    };

    for (int batch = 0; batch < n_batches; ++batch) {
        const int j0 = batch * kSlotBatch;
        const int nj = (level == 0) ? a.J : ((a.J - j0 < kSlotBatch) ? a.J - j0 : kSlotBatch);
        const int n_hist = (level == 0) ? 1 : nj;
        list_j0 = j0;
        long long cur_group = -1;
        for (u64 cb = c0; cb < c1; cb += n_sub) {         // uniform over the workgroup
            // wide workgroups run under GLOBAL scope only, where every chunk belongs to group 0
            const long long g = a.per_tensor ? static_cast<long long>(a.chunk_map[cb]) : 0;
            if (g != cur_group) {
                if (cur_group >= 0) {                     // flush the previous group's counts
                    __syncthreads();
                    flush(cur_group, j0, n_hist);
                }
                __syncthreads();
                if (wtid == 0) s_any = 0;
                __syncthreads();
                if (level == 0) {
                    if (wtid < a.J && a.slots[g * a.J + wtid].state == kSelecting) s_any = 1;
                } else if (wtid < nj && a.merged) {
                    s_prefix[wtid] = s_mprefix[j0 + wtid];
                    s_active[wtid] = s_mactive[j0 + wtid];
                    if (s_active[wtid]) s_any = 1;
                } else if (wtid < nj) {
                    const Slot& s = a.slots[g * a.J + j0 + wtid];
                    s_prefix[wtid] = static_cast<u32>(s.prefix);
                    s_active[wtid] = (s.state == kSelecting) ? 1u : 0u;
                    if (s.state == kSelecting) s_any = 1;
                }
                for (int i = wtid; i < n_hist * nb; i += wide) s_hist[i] = 0;
                if (level != 0) for (int i = wtid; i < kBins; i += wide) s_tab[i] = 0;
                __syncthreads();
                if (level != 0 && wtid == 0)
                    for (int j = 0; j < nj; ++j)
                        if (s_active[j]) s_tab[s_prefix[j] >> L0.shift] |= static_cast<u16>(1u << j);
                __syncthreads();
                cur_group = g;
            }
            if (!s_any) continue;
            single = (level != 0 && nj == 1);             // its ranking is selecting, or s_any would be 0
            p0 = single ? s_prefix[0] : 0u;
            const u64 c = cb + sub;
            if (c >= c1) continue;                        // no barrier below this point in the iteration
            hit = a.tiehit + c;
            const int t = static_cast<int>(a.chunk_map[c]);
            const TensorDesc& td = a.td[t];
            const u64 base = (c - td.chunk_start) * kChunk;
            const u64 n = td.n;
            chunk_flat = td.flat_start + base;
            if (VEC && base + kChunk <= n) {              // whole chunk inside the tensor: loads first
                constexpr int kHalf = LC ? kQuadsPerThread / 2 : kQuadsPerThread;
#pragma unroll
                for (int h = 0; h < kQuadsPerThread / kHalf; ++h) {
                    float4 wv[kHalf], lv[kHalf];
#pragma unroll
                    for (int q = 0; q < kHalf; ++q) {
                        const u64 e0 = base + static_cast<u64>(h * kHalf + q) * (kBlock * 4) + tid * 4;
                        wv[q] = a.streaming ? ld4_stream(td.w + e0) : *reinterpret_cast<const float4*>(td.w + e0);
                        if (LC) lv[q] = a.streaming ? ld4_stream(td.lam + e0) : *reinterpret_cast<const float4*>(td.lam + e0);
                    }
#pragma unroll
                    for (int q = 0; q < kHalf; ++q) {
                        float v[4] = {wv[q].x, wv[q].y, wv[q].z, wv[q].w};
                        if (LC) {
                            const float l[4] = {lv[q].x, lv[q].y, lv[q].z, lv[q].w};
#pragma unroll
                            for (int k = 0; k < 4; ++k) v[k] = lc_shift(v[k], l[k], a.mu);
                        }
#pragma unroll
                        for (int k = 0; k < 4; ++k)
                            count_key(mag_key(v[k]), static_cast<u32>((h * kHalf + q) * (kBlock * 4) + tid * 4 + k));
                    }
                }
            } else {
                for (int q = 0; q < kQuadsPerThread; ++q) {
                    const u64 e0 = base + static_cast<u64>(q) * (kBlock * 4) + tid * 4;
                    if (e0 >= n) break;
                    float v[4];
                    load4<VEC>(td.w, e0, n, v);
                    if (LC) {
                        float l[4];
                        load4<VEC>(td.lam, e0, n, l);
#pragma unroll
                        for (int k = 0; k < 4; ++k) v[k] = lc_shift(v[k], l[k], a.mu);
                    }
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        if (e0 + k >= n) break;
                        count_key(mag_key(v[k]), static_cast<u32>(e0 - base) + k);
                    }
                }
            }
        }
        if (cur_group >= 0) {
            __syncthreads();
            flush(cur_group, j0, n_hist);
            __syncthreads();
        }
    }
    if (listing) {                                         // hand the buffered entries to the rankings' lists
        __syncthreads();
        const u32 n_l = s_ln;                              // uniform
        if (n_l > kTieListGroup) {
            if (wtid < a.J)
                atomicAdd(reinterpret_cast<unsigned long long*>(&a.tl_cnt[wtid]), static_cast<unsigned long long>(kTieListCap) + 1);
        } else if (n_l > 0) {
            if (wtid < a.J) {                              // one reservation per ranking
                u32 mine = 0;
                for (u32 i = 0; i < n_l; ++i) mine += (s_lj[i] == static_cast<u32>(wtid)) ? 1u : 0u;
                s_lbase[wtid] = mine ? atomicAdd(reinterpret_cast<unsigned long long*>(&a.tl_cnt[wtid]), static_cast<unsigned long long>(mine)) : 0;
            }
            __syncthreads();
            if (static_cast<u32>(wtid) < n_l) {            // a workgroup has at least 256 threads, a buffer 128 entries
                const u32 j = s_lj[wtid];
                u32 before = 0;
                for (int i = 0; i < wtid; ++i) before += (s_lj[i] == j) ? 1u : 0u;
                const u64 pos = s_lbase[j] + before;
                if (pos < kTieListCap) {
                    a.tl_key[static_cast<u64>(j) * kTieListCap + pos] = s_lkey[wtid];
                    a.tl_idx[static_cast<u64>(j) * kTieListCap + pos] = s_lidx[wtid];
                }
            }
        }
    }
}

// ---- one level of the search: locate the bin that holds the wanted rank -------------------------
//
// One workgroup per ranking.  Bins are walked from the top; the bin b with
//   #(keys in higher bins) < remaining <= #(keys in bins >= b)
// extends the prefix.  After the last level the prefix is the threshold key, `remaining` the number
// of ties to keep and n_tie the number of keys equal to the threshold.
__global__ __launch_bounds__(kBlock) void k_scan_level(Slot* slots, const u64* hist_shared, u64* hist_slot,
                                                       int J, int key_bits, int level, Control* ctl,
                                                       int only_failed, u32* tie_flag) {
    __shared__ u64 s_wave[kBlock / 64];
    if (only_failed && ctl->window_failed == 0) return;
    const int s = blockIdx.x;
    Slot& slot = slots[s];
    if (slot.state != kSelecting) return;             // uniform over the workgroup
    if (static_cast<u32>(level) < slot.level_begin) return;
    const Level L = level_of(key_bits, level);
    const int nb = 1 << L.bits;
    const bool shared = (level == 0 && hist_shared != nullptr);
    const u64* hist = shared ? hist_shared + static_cast<u64>(s / J) * kBins : hist_slot + static_cast<u64>(s) * kBins;
    constexpr int kPer = kBins / kBlock;              // 8 bins per thread, from the top
    const int tid = threadIdx.x;
    u64 cnt[kPer];
    u64 sum = 0;
#pragma unroll
    for (int i = 0; i < kPer; ++i) {
        const int b = nb - 1 - (tid * kPer + i);
        cnt[i] = (b >= 0) ? hist[b] : 0;
        sum += cnt[i];
    }
    const u64 remaining = slot.remaining;
    u64 total;
    u64 cum = block_excl_scan_u64(sum, s_wave, &total);
    __syncthreads();                                   // every thread has read slot.remaining
#pragma unroll
    for (int i = 0; i < kPer; ++i) {
        const int b = nb - 1 - (tid * kPer + i);
        if (b >= 0 && cum < remaining && remaining <= cum + cnt[i]) {
            const u64 rem = remaining - cum;
            slot.prefix |= static_cast<u64>(b) << L.shift;
            slot.remaining = rem;
            slot.n_tie = cnt[i];
            if (level == n_levels(key_bits) - 1) {
                slot.state = kDone;
                if (rem < cnt[i]) {
                    slot.need_tie = 1;
                    atomicOr(tie_flag, 1u);
                } else {
                    slot.need_tie = 0;
                    slot.tie_end = slot.n;
                }
            }
        }
        cum += cnt[i];
    }
    if (tid == 0 && total < remaining) {               // the wanted rank is not in this population
        slot.state = kFailed;
        atomicOr(&ctl->window_failed, 1u);
    }
    if (!shared) {                                     // leave the ranking's histogram clean for the next level
        u64* h = hist_slot + static_cast<u64>(s) * kBins;
        for (int i = tid; i < nb; i += kBlock) h[i] = 0;
    }
}

// ---- ties: count per chunk, then find the chunk and the element that ends the kept ties ---------

template <bool LC, bool VEC>
__global__ __launch_bounds__(kBlock) void k_tie_count(DataArgs a) {
    __shared__ u16 s_tab[kBins];
    __shared__ u32 s_T[kMaxJ];
    __shared__ u32 s_need[kMaxJ];
    __shared__ u32 s_cnt[kMaxJ];
    __shared__ u32 s_mT[kMaxJ];           // merged form: thresholds and tie needs after the last level
    __shared__ u32 s_mneed[kMaxJ];
    __shared__ u32 s_any;
    if (a.only_failed && a.ctl->window_failed == 0) return;
    if (a.merged) {
        const int last = n_levels(31) - 1;
        if (threadIdx.x == 0) s_any = 0;
        __syncthreads();
        for (int j = static_cast<int>(threadIdx.x) >> 6; j < a.J; j += kBlock / 64) {
            const u64* prev = last == 0 ? a.hist0 : data_hist(a, last, j);
            const SlotStep e = wave_enter_level(a.slots[j], last + 1, 31, prev, coarse_of(a.hist0, a.coarse, prev));
            if ((threadIdx.x & 63) == 0) {
                s_mT[j] = static_cast<u32>(e.prefix);
                // rankings whose ties are all in their short list are finished by k_tie_locate alone
                s_mneed[j] = (e.state == kDone && e.need_tie && !tie_list_usable(a, j, e.n_tie)) ? 1u : 0u;
                if (s_mneed[j]) s_any = 1;
            }
        }
        __syncthreads();
        if (!s_any) return;               // uniform: no ranking keeps only part of its ties
        __syncthreads();
    } else if (a.ctl->need_tie == 0) return;
    const Level L0 = level_of(31, 0);
    const int tid = threadIdx.x;
    long long cur_group = -1;
    auto count_key = [&](u32 key) {
        u32 m = s_tab[key >> L0.shift];
        while (m) {
            const int j = __ffs(m) - 1;
            m &= m - 1;
            if (key == s_T[j]) atomicAdd(&s_cnt[j], 1u);
        }
    };
    for (u64 c = blockIdx.x; c < a.n_chunks; c += gridDim.x) {
        if (a.tiehit[c] == 0) continue;                   // uniform: no key of this chunk reached the last level's bins,
                                                          // so it holds no tie and its count stays at the cleared 0
        const int t = static_cast<int>(a.chunk_map[c]);
        const long long g = a.per_tensor ? t : 0;
        __syncthreads();
        if (g != cur_group) {
            if (tid == 0) s_any = 0;
            __syncthreads();
            if (tid < a.J && a.merged) {
                s_T[tid] = s_mT[tid];
                s_need[tid] = s_mneed[tid];
                if (s_need[tid]) s_any = 1;
            } else if (tid < a.J) {
                const Slot& s = a.slots[static_cast<u64>(g) * a.J + tid];
                s_T[tid] = static_cast<u32>(s.prefix);
                s_need[tid] = (s.state == kDone && s.need_tie) ? 1u : 0u;
                if (s_need[tid]) s_any = 1;
            }
            __syncthreads();
            build_digit_table(s_tab, s_T, s_need, a.J, tid);
            cur_group = g;
        }
        if (tid < a.J) s_cnt[tid] = 0;
        __syncthreads();
        if (!s_any) continue;
        const TensorDesc& td = a.td[t];
        const u64 base = (c - td.chunk_start) * kChunk;
        const u64 n = td.n;
        if (VEC && base + kChunk <= n) {
            constexpr int kHalf = LC ? kQuadsPerThread / 2 : kQuadsPerThread;
#pragma unroll
            for (int h = 0; h < kQuadsPerThread / kHalf; ++h) {
                float4 wv[kHalf], lv[kHalf];
#pragma unroll
                for (int q = 0; q < kHalf; ++q) {
                    const u64 e0 = base + static_cast<u64>(h * kHalf + q) * (kBlock * 4) + tid * 4;
                    wv[q] = a.streaming ? ld4_stream(td.w + e0) : *reinterpret_cast<const float4*>(td.w + e0);
                    if (LC) lv[q] = a.streaming ? ld4_stream(td.lam + e0) : *reinterpret_cast<const float4*>(td.lam + e0);
                }
#pragma unroll
                for (int q = 0; q < kHalf; ++q) {
                    float v[4] = {wv[q].x, wv[q].y, wv[q].z, wv[q].w};
                    if (LC) {
                        const float l[4] = {lv[q].x, lv[q].y, lv[q].z, lv[q].w};
#pragma unroll
                        for (int k = 0; k < 4; ++k) v[k] = lc_shift(v[k], l[k], a.mu);
                    }
#pragma unroll
                    for (int k = 0; k < 4; ++k) count_key(mag_key(v[k]));
                }
            }
        } else {
            for (int q = 0; q < kQuadsPerThread; ++q) {
                const u64 e0 = base + static_cast<u64>(q) * (kBlock * 4) + tid * 4;
                if (e0 >= n) break;
                float v[4];
                load4<VEC>(td.w, e0, n, v);
                if (LC) {
                    float l[4];
                    load4<VEC>(td.lam, e0, n, l);
#pragma unroll
                    for (int k = 0; k < 4; ++k) v[k] = lc_shift(v[k], l[k], a.mu);
                }
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    if (e0 + k >= n) break;
                    count_key(mag_key(v[k]));
                }
            }
        }
        __syncthreads();
        if (tid < a.J && s_need[tid]) a.tiecnt[static_cast<u64>(tid) * a.n_chunks + c] = s_cnt[tid];
    }
}
template <bool LC, bool VEC>
__global__ __launch_bounds__(kBlock) void k_tie_locate(DataArgs a, condensa_select* results, int n_groups) {
    __shared__ u64 s_wave[kBlock / 64];
    __shared__ u64 s_found[3];                 // chunk, rank inside it, flag
    __shared__ u64 s_run[3];                   // run of chunks that holds the wanted tie, ties before the run
    __shared__ SlotStep s_e;
    const int s = blockIdx.x;
    const int g = s / a.J, j = s % a.J;
    const int tid = threadIdx.x;
    Slot& slot = a.slots[s];
    if (a.merged) {
        // the last level's histogram is folded in here, and this workgroup (the only one that touches the
        // ranking in this kernel) makes the outcome the ranking's stored state
        if (tid < 64) {
            const int last = n_levels(31) - 1;
            const u64* prev = last == 0 ? a.hist0 : data_hist(a, last, s);
            const SlotStep e = wave_enter_level(slot, last + 1, 31, prev, coarse_of(a.hist0, a.coarse, prev));
            if (tid == 0) {
                s_e = e;
                if (slot.state == kSelecting) {
                    slot.prefix = e.prefix; slot.remaining = e.remaining; slot.n_tie = e.n_tie;
                    slot.state = e.state; slot.need_tie = e.need_tie;
                    if (e.state == kDone && !e.need_tie) slot.tie_end = slot.n;
                }
            }
        }
    } else if (tid == 0) {
        s_e = slot_canonical(slot);
    }
    __syncthreads();
    const bool need = (s_e.state == kDone && s_e.need_tie);
    const bool from_list = need && a.merged && tie_list_usable(a, j, s_e.n_tie);     // uniform
    if (from_list) {
        // The ties are among the few keys that the last level listed: gather their flat indices in LDS and
        // rank each by counting the lower ones (flat indices are distinct, so exactly one has rank r).
        __shared__ u64 s_tie[kTieListTies];
        __shared__ u32 s_n;
        const u64 r = s_e.remaining;
        const u32 T = static_cast<u32>(s_e.prefix);
        const u32 n_list = static_cast<u32>(a.tl_cnt[j]);
        if (tid == 0) s_n = 0;
        __syncthreads();
        for (u32 i = tid; i < n_list; i += kBlock)
            if (a.tl_key[static_cast<u64>(j) * kTieListCap + i] == T) {
                const u32 pos = atomicAdd(&s_n, 1u);
                if (pos < kTieListTies) s_tie[pos] = a.tl_idx[static_cast<u64>(j) * kTieListCap + i];
            }
        __syncthreads();
        const u32 m = s_n < kTieListTies ? s_n : kTieListTies;
        for (u32 i = tid; i < m; i += kBlock) {
            const u64 mine = s_tie[i];
            u64 lower = 0;
            for (u32 e = 0; e < m; ++e) lower += (s_tie[e] < mine) ? 1u : 0u;
            if (lower + 1 == r) slot.tie_end = mine + 1;
        }
        __syncthreads();
    } else if (need) {
        const u64 r = s_e.remaining;           // 1-based rank of the last kept tie
        const u32 T = static_cast<u32>(s_e.prefix);
        const u64 cb = a.per_tensor ? a.td[g].chunk_start : 0;
        const u64 ce = a.per_tensor ? a.td[g + 1].chunk_start : a.n_chunks;
        const u32* cnt = a.tiecnt + static_cast<u64>(j) * a.n_chunks;
        // every thread owns a contiguous run of the chunk range
        const u64 per = (ce - cb + kBlock - 1) / kBlock;
        const u64 my0 = cb + per * tid < ce ? cb + per * tid : ce;
        const u64 my1 = my0 + per < ce ? my0 + per : ce;
        u64 mine = 0;
        for (u64 c = my0; c < my1; c += 8) {          // eight loads in flight: the loop waits on latency only
            u32 x[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) x[u] = (c + u < my1) ? cnt[c + u] : 0u;
#pragma unroll
            for (int u = 0; u < 8; ++u) mine += x[u];
        }
        u64 total;
        u64 before = block_excl_scan_u64(mine, s_wave, &total);
        if (tid == 0) s_found[2] = 0;
        __syncthreads();
        // the thread whose run holds the r-th tie publishes the run; the workgroup then searches it together
        if (before < r && r <= before + mine) { s_run[0] = my0; s_run[1] = my1; s_run[2] = before; s_found[2] = 2; }
        __syncthreads();
        if (s_found[2] == 2) {
            const u64 run0 = s_run[0], run1 = s_run[1];
            u64 cum = s_run[2];
            __syncthreads();
            for (u64 i0 = run0; i0 < run1; i0 += kBlock) {                 // uniform trip count
                const u64 c = i0 + tid;
                const u64 x = (c < run1) ? cnt[c] : 0;
                u64 tot;
                const u64 ex = block_excl_scan_u64(x, s_wave, &tot);
                if (cum + ex < r && r <= cum + ex + x) { s_found[0] = c; s_found[1] = r - (cum + ex); s_found[2] = 1; }
                cum += tot;
            }
        }
        __syncthreads();
        if (s_found[2] == 2) s_found[2] = 0;          // cannot happen: the run's counts add up to `mine`
        __syncthreads();
        if (s_found[2]) {
            const u64 c = s_found[0];
            const u64 rr = s_found[1];
            const int t = static_cast<int>(a.chunk_map[c]);
            const TensorDesc& td = a.td[t];
            const u64 base = (c - td.chunk_start) * kChunk;
            constexpr int kRun = kChunk / kBlock;              // 32 consecutive elements per thread
            const u64 e_begin = base + static_cast<u64>(tid) * kRun;
            // bit k of `eq`: element e_begin + k exists and its key equals T (all loads issued before the first use)
            u32 eq = 0;
            if (VEC && e_begin + kRun <= td.n) {
                float4 wv[kRun / 4], lv[kRun / 4];
#pragma unroll
                for (int q = 0; q < kRun / 4; ++q) {
                    wv[q] = *reinterpret_cast<const float4*>(td.w + e_begin + 4 * q);
                    if (LC) lv[q] = *reinterpret_cast<const float4*>(td.lam + e_begin + 4 * q);
                }
#pragma unroll
                for (int q = 0; q < kRun / 4; ++q) {
                    float v[4] = {wv[q].x, wv[q].y, wv[q].z, wv[q].w};
                    if (LC) {
                        const float l[4] = {lv[q].x, lv[q].y, lv[q].z, lv[q].w};
#pragma unroll
                        for (int k = 0; k < 4; ++k) v[k] = lc_shift(v[k], l[k], a.mu);
                    }
#pragma unroll
                    for (int k = 0; k < 4; ++k) eq |= (mag_key(v[k]) == T ? 1u : 0u) << (4 * q + k);
                }
            } else {
                for (int k = 0; k < kRun; ++k) {
                    const u64 e = e_begin + k;
                    if (e >= td.n) break;
                    const float x = LC ? lc_shift(td.w[e], td.lam[e], a.mu) : td.w[e];
                    eq |= (mag_key(x) == T ? 1u : 0u) << k;
                }
            }
            const u32 hits = __popc(eq);
            u64 tot2;
            const u64 bef2 = block_excl_scan_u64(hits, s_wave, &tot2);
            if (bef2 < rr && rr <= bef2 + hits) {
                u32 m = eq;
                for (u64 skip = rr - bef2 - 1; skip > 0; --skip) m &= m - 1;      // drop the ties before the wanted one
                slot.tie_end = (a.per_tensor ? 0 : td.flat_start) + e_begin + (__ffs(m) - 1) + 1;
            }
        }
        __syncthreads();
    }
    __threadfence_block();
    __syncthreads();
    if (tid == 0) {
        condensa_select out;
        out.n = slot.n;
        out.k = slot.k;
        if (s_e.state == kDone) {
            out.n_gt = slot.k - s_e.remaining;
            out.n_tie_kept = s_e.remaining;
            out.n_tie = s_e.n_tie;
            out.threshold_key = s_e.prefix;
            out.tie_end = slot.tie_end;
        } else {                                  // k == 0: nothing is kept
            out.n_gt = 0; out.n_tie_kept = 0; out.n_tie = 0;
            out.threshold_key = ~static_cast<u64>(0);
            out.tie_end = 0;
        }
        out.path = slot.path;
        results[static_cast<u64>(j) * n_groups + g] = out;
    }
}

}  // namespace condensa
