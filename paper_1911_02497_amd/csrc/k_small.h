// Small calls (up to kSmallCallElems elements, GLOBAL scope): two launches after the first radix level.
//
// A call on a single layer or a small model is bound by its launches: three histogram sweeps, the tie sweep
// and the tie search are five dependent launches around a few microseconds of work each.  After the first
// level (11 of 31 key bits) the bins that hold the thresholds contain a few percent of the keys at most, so
// the second sweep lists those keys with their flat indices instead of counting them (k_small_collect), and
// one workgroup per ranking finishes on the list: the two remaining levels, the tie rule and the result
// record (k_small_finish).  The list can hold every element of the call, so nothing can overflow: a
// degenerate input (all keys in one bin) is only slower, never wrong.
// Section 3.1 (a sparsity turned into a magnitude threshold); Results (up to ten samples per search).
#pragma once
#include "k_select.h"

namespace condensa {

constexpr u64 kSmallCallElems = static_cast<u64>(1) << 21;
constexpr int kSmallFinishThreads = 1024;

// Wavefront 0 of a workgroup: the bin of an LDS histogram (nb <= kBins bins) that holds descending rank r, i.e.
// #(keys in higher bins) < r <= #(keys in bins >= bin).  The lane that finds it writes bin, the rank inside
// the bin, the bin's count and *found = 1; nothing is written when the histogram holds fewer than r keys.
__device__ inline void wave_pick_desc(const u32* s_hist, int nb, u64 r, u32* bin, u64* rem, u64* cnt, u32* found) {
    constexpr int kPerMax = kBins / 64;
    const int lane = threadIdx.x & 63;
    const int per = (nb + 63) / 64;
    u32 c[kPerMax];
    u64 sum = 0;
#pragma unroll
    for (int i = 0; i < kPerMax; ++i) {
        const int b = nb - 1 - (lane * per + i);
        c[i] = (i < per && b >= 0) ? s_hist[b] : 0u;
        sum += c[i];
    }
    const u64 incl = wave_incl_scan_u64(sum);
    u64 before = incl - sum;
    if (before < r && r <= incl) {
#pragma unroll
        for (int i = 0; i < kPerMax; ++i) {
            if (before < r && r <= before + c[i]) {
                *bin = static_cast<u32>(nb - 1 - (lane * per + i));
                *rem = r - before;
                *cnt = c[i];
                *found = 1u;
            }
            before += c[i];
        }
    }
}

// The same for ascending rank r (the r-th lowest), used for the index search among ties.
__device__ inline void wave_pick_asc(const u32* s_hist, int nb, u64 r, u32* bin, u64* rem, u32* found) {
    constexpr int kPerMax = kBins / 64;
    const int lane = threadIdx.x & 63;
    const int per = (nb + 63) / 64;
    u32 c[kPerMax];
    u64 sum = 0;
#pragma unroll
    for (int i = 0; i < kPerMax; ++i) {
        const int b = lane * per + i;
        c[i] = (i < per && b < nb) ? s_hist[b] : 0u;
        sum += c[i];
    }
    const u64 incl = wave_incl_scan_u64(sum);
    u64 before = incl - sum;
    if (before < r && r <= incl) {
#pragma unroll
        for (int i = 0; i < kPerMax; ++i) {
            if (before < r && r <= before + c[i]) {
                *bin = static_cast<u32>(lane * per + i);
                *rem = r - before;
                *found = 1u;
            }
            before += c[i];
        }
    }
}

// Second sweep of a small call: every workgroup folds in level 0 for each ranking, then appends the (key, flat
// index) of every key whose leading digit is the leading digit of some threshold to the call's list
// (tl_key / tl_idx, counter tl_cnt[0]).  One reservation per workgroup and chunk; the order of the list does not
// matter to what is computed from it.
template <bool LC, bool VEC>
__global__ __launch_bounds__(kBlock) void k_small_collect(DataArgs a) {
    __shared__ u16 s_tab[kBins];
    __shared__ u32 s_prefix[kMaxJ];
    __shared__ u32 s_active[kMaxJ];
    __shared__ u64 s_wave[kBlock / 64];
    __shared__ u64 s_base;
    const int tid = threadIdx.x;
    for (int j = tid >> 6; j < a.J; j += kBlock / 64) {
        const SlotStep e = wave_enter_level(a.slots[j], 1, 31, a.hist0, coarse_of(a.hist0, a.coarse, a.hist0));
        if ((tid & 63) == 0) {
            s_prefix[j] = static_cast<u32>(e.prefix);
            s_active[j] = (e.state == kSelecting) ? 1u : 0u;
        }
    }
    __syncthreads();
    build_digit_table(s_tab, s_prefix, s_active, a.J, tid);
    __syncthreads();
    const Level L0 = level_of(31, 0);
    for (u64 c = blockIdx.x; c < a.n_chunks; c += gridDim.x) {
        const int t = static_cast<int>(a.chunk_map[c]);
        const TensorDesc& td = a.td[t];
        const u64 base = (c - td.chunk_start) * kChunk;
        const u64 n = td.n;
        u32 key[kQuadsPerThread * 4];
        u32 listed = 0;                                    // bit q * 4 + k: element q * 1024 + tid * 4 + k of the chunk
        if (VEC && base + kChunk <= n) {                   // whole chunk inside the tensor: loads first
            constexpr int kHalf = LC ? kQuadsPerThread / 2 : kQuadsPerThread;
#pragma unroll
            for (int h = 0; h < kQuadsPerThread / kHalf; ++h) {
                float4 wv[kHalf], lv[kHalf];
#pragma unroll
                for (int q = 0; q < kHalf; ++q) {
                    const u64 e0 = base + static_cast<u64>(h * kHalf + q) * (kBlock * 4) + tid * 4;
                    wv[q] = *reinterpret_cast<const float4*>(td.w + e0);
                    if (LC) lv[q] = *reinterpret_cast<const float4*>(td.lam + e0);
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
                    for (int k = 0; k < 4; ++k) {
                        const int i = (h * kHalf + q) * 4 + k;
                        key[i] = mag_key(v[k]);
                        if (s_tab[key[i] >> L0.shift] != 0) listed |= 1u << i;
                    }
                }
            }
        } else {
#pragma unroll
            for (int q = 0; q < kQuadsPerThread; ++q) {
                const u64 e0 = base + static_cast<u64>(q) * (kBlock * 4) + tid * 4;
                float v[4] = {0.0f, 0.0f, 0.0f, 0.0f};
                if (e0 < n) {
                    load4<VEC>(td.w, e0, n, v);
                    if (LC) {
                        float l[4];
                        load4<VEC>(td.lam, e0, n, l);
#pragma unroll
                        for (int k = 0; k < 4; ++k) v[k] = lc_shift(v[k], l[k], a.mu);
                    }
                }
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const int i = q * 4 + k;
                    key[i] = mag_key(v[k]);
                    if (e0 + k < n && s_tab[key[i] >> L0.shift] != 0) listed |= 1u << i;
                }
            }
        }
        u64 total;
        const u64 before = block_excl_scan_u64(static_cast<u64>(__popc(listed)), s_wave, &total);
        if (total != 0) {                                  // uniform over the workgroup
            if (tid == 0) s_base = atomicAdd(reinterpret_cast<unsigned long long*>(&a.tl_cnt[0]), static_cast<unsigned long long>(total));
            __syncthreads();
            u64 pos = s_base + before;
#pragma unroll
            for (int i = 0; i < kQuadsPerThread * 4; ++i) {
                if (listed & (1u << i)) {
                    if (pos < a.small_cap) {
                        a.tl_key[pos] = key[i];
                        a.tl_idx[pos] = td.flat_start + base + static_cast<u64>(i / 4) * (kBlock * 4) + tid * 4 + (i % 4);
                    }
                    ++pos;
                }
            }
            __syncthreads();                               // s_base is rewritten for the next chunk
        }
    }
}

// A 1024-thread workgroup finishes one ranking on a list of (key, index) entries that holds every key sharing the
// ranking's digits above `first_level` (and possibly other keys): `e` is the ranking's state on entering that
// level.  The remaining levels are counted in LDS over the matching entries, the tie rule picks the r-th lowest
// index among the entries equal to the threshold, and the outcome becomes the ranking's stored state and its
// result record.  Called by every thread of the workgroup with the same arguments.
template <typename KEY, typename IDX>
__device__ inline void finish_on_list(Slot& slot, SlotStep e, const KEY* __restrict__ keys, const IDX* __restrict__ ids,
                                      u64 n_list, int key_bits, int first_level, int idx_bits, condensa_select* record) {
    __shared__ __align__(8) u32 s_hist[kBins];
    __shared__ u32 s_bin, s_found, s_n;
    __shared__ u64 s_rem, s_cnt;
    const int tid = threadIdx.x;
    u64 tie_end = slot.n;                                  // every tie kept, unless found otherwise below
    if (e.state == kSelecting) {                           // uniform over the workgroup
        u64 prefix = e.prefix, r = e.remaining, n_tie = 0;
        bool ok = true;
        for (int level = first_level; level < n_levels(key_bits) && ok; ++level) {
            const Level lv = level_of(key_bits, level);
            const int nb = 1 << lv.bits;
            for (int i = tid; i < nb; i += kSmallFinishThreads) s_hist[i] = 0;
            if (tid == 0) s_found = 0;
            __syncthreads();
            for (u64 i = tid; i < n_list; i += kSmallFinishThreads) {
                const u64 key = keys[i];
                if (((key ^ prefix) >> lv.hi_shift) == 0) atomicAdd(&s_hist[static_cast<u32>(key >> lv.shift) & (nb - 1)], 1u);
            }
            __syncthreads();
            if (tid < 64) wave_pick_desc(s_hist, nb, r, &s_bin, &s_rem, &s_cnt, &s_found);
            __syncthreads();
            ok = s_found != 0;
            if (ok) {
                prefix |= static_cast<u64>(s_bin) << lv.shift;
                r = s_rem;
                n_tie = s_cnt;
            }
            __syncthreads();
        }
        if (!ok) {
            e.state = kFailed;                             // the counts of the levels and the list disagree: reported, not hidden
        } else {
            e.prefix = prefix; e.remaining = r; e.n_tie = n_tie; e.state = kDone; e.need_tie = 0;
            const u64 T = prefix;
            if (r < n_tie && n_tie <= static_cast<u64>(kSmallFinishThreads)) {
                // a handful of ties: their indices in LDS, each ranked by counting the lower ones
                u64* s_idx = reinterpret_cast<u64*>(s_hist);
                if (tid == 0) { s_n = 0; s_rem = slot.n - 1; }
                __syncthreads();
                for (u64 i = tid; i < n_list; i += kSmallFinishThreads)
                    if (static_cast<u64>(keys[i]) == T) {
                        const u32 p = atomicAdd(&s_n, 1u);
                        if (p < static_cast<u32>(kSmallFinishThreads)) s_idx[p] = static_cast<u64>(ids[i]);
                    }
                __syncthreads();
                const u32 m = s_n < static_cast<u32>(kSmallFinishThreads) ? s_n : static_cast<u32>(kSmallFinishThreads);
                if (static_cast<u32>(tid) < m) {
                    const u64 mine = s_idx[tid];
                    u64 lower = 0;
                    for (u32 i = 0; i < m; ++i) lower += (s_idx[i] < mine) ? 1u : 0u;
                    if (lower + 1 == r) s_rem = mine;      // indices are distinct: one thread
                }
                __syncthreads();
                tie_end = s_rem + 1;
            } else if (r < n_tie) {
                // many ties: radix levels on the index over the entries equal to the threshold, lowest first
                u64 iprefix = 0, ir = r;
                for (int level = 0; level < n_levels(idx_bits); ++level) {     // uniform
                    const Level lv = level_of(idx_bits, level);
                    const int nb = 1 << lv.bits;
                    for (int i = tid; i < nb; i += kSmallFinishThreads) s_hist[i] = 0;
                    if (tid == 0) s_found = 0;
                    __syncthreads();
                    for (u64 i = tid; i < n_list; i += kSmallFinishThreads) {
                        if (static_cast<u64>(keys[i]) != T) continue;
                        const u64 idx = static_cast<u64>(ids[i]);
                        if (((idx ^ iprefix) >> lv.hi_shift) == 0) atomicAdd(&s_hist[static_cast<u32>(idx >> lv.shift) & (nb - 1)], 1u);
                    }
                    __syncthreads();
                    if (tid < 64) wave_pick_asc(s_hist, nb, ir, &s_bin, &s_rem, &s_found);
                    __syncthreads();
                    iprefix |= static_cast<u64>(s_bin) << lv.shift;
                    ir = s_rem;
                    __syncthreads();
                }
                tie_end = iprefix + 1;
            }
        }
    }
    if (tid != 0) return;
    if (slot.state == kSelecting) {
        slot.prefix = e.prefix; slot.remaining = e.remaining; slot.n_tie = e.n_tie;
        slot.state = e.state; slot.need_tie = 0;
        slot.tie_end = tie_end;
    }
    condensa_select out;
    out.n = slot.n;
    out.k = slot.k;
    if (e.state == kDone) {
        out.n_gt = slot.k - e.remaining;
        out.n_tie_kept = e.remaining;
        out.n_tie = e.n_tie;
        out.threshold_key = e.prefix;
        out.tie_end = slot.tie_end;
    } else {                                               // k == 0: nothing is kept
        out.n_gt = 0; out.n_tie_kept = 0; out.n_tie = 0;
        out.threshold_key = ~static_cast<u64>(0);
        out.tie_end = 0;
    }
    out.path = slot.path;
    *record = out;
}

// One workgroup per ranking: level 0 is folded in, the rest happens on the list.
__global__ __launch_bounds__(kSmallFinishThreads) void k_small_finish(DataArgs a, condensa_select* results, int idx_bits) {
    __shared__ SlotStep s_e;
    const int j = blockIdx.x;
    Slot& slot = a.slots[j];
    if (threadIdx.x < 64) {
        const SlotStep e = wave_enter_level(slot, 1, 31, a.hist0, coarse_of(a.hist0, a.coarse, a.hist0));
        if (threadIdx.x == 0) s_e = e;
    }
    __syncthreads();
    u64 n_list = a.tl_cnt[0];
    if (n_list > a.small_cap) n_list = a.small_cap;        // (cannot happen: the list holds every element)
    finish_on_list<u32, u64>(slot, s_e, a.tl_key, a.tl_idx, n_list, 31, 1, idx_bits, results + j);
}

}  // namespace condensa
