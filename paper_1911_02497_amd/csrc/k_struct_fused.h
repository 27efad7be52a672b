// BlockPrune (Table 1) with the weights read once: aggregation and apply in one sweep for 8x8 blocks.
//
// Structure pruning needs every aggregate before the first block can be decided, so the plain form reads
// the weights twice (aggregate, then apply: 13 bytes per weight with theta and mask).  As for element
// pruning, a sample supplies a prior: the aggregates of a sample of blocks are ranked, the sample ranks
// around the expected position of the threshold bound a window [lo, hi] on the aggregates, and the sweep
// that computes the aggregates already writes the final theta and mask of every block outside the window
// (kept above hi, zeroed below lo) -- an 8x8 block sits in the registers of the thread that adds it up.
// Blocks inside the window get a provisional decision (kept iff above `mid`, the sample's estimate of the
// threshold) and are listed with their aggregates.  The sweep also counts the blocks above the window, so the
// exact ranking only has to find rank k - above among the listed blocks (a percent of all blocks) instead of
// rank k among all of them; when that rank does not fall inside the list, or the list overflowed, the ranking
// over all stored aggregates runs as in the plain form and a gated full apply sweep rewrites everything.
// Threshold, tie rule, structure mask and kept-id list never depend on the sample.  A fix-up pass rewrites the
// listed blocks whose final decision differs from the provisional one.  9.3 instead of 13 bytes per weight.
#pragma once
#include "k_structure.h"
#include "k_window.h"

namespace condensa {

struct StructWindowArgs {
    u32* sample;           // [n_units] upper 31 bits of the sampled blocks' aggregates
    u64 n_units;
    u64 stride;            // one sampled block per stride of structures
    Slot* wslots;          // [3] boundary rankings of the sample: upper bound, lower bound, estimate
    u64* seg_cnt;          // [kSegs] listed blocks per segment (may exceed seg_cap)
    u64* seg_above;        // [kSegs] blocks above the window
    u32* cand_id;          // [n_segs][seg_cap] ids of the blocks inside the window
    u64* cand_key;         // [n_segs][seg_cap] their aggregate keys
    u64 seg_cap;
    u32 n_segs;
    const OutDesc* out;
};

// The window on the 63-bit aggregate patterns from the 31-bit bounds that the sample ranking left.
__device__ inline u64 window_lo63(const Slot* ws) { return ws[1].prefix << 32; }
__device__ inline u64 window_hi63(const Slot* ws) { return (ws[0].prefix << 32) | 0xFFFFFFFFull; }
__device__ inline u64 window_mid63(const Slot* ws) {
    const u64 lo = ws[1].prefix, hi = ws[0].prefix, m = ws[2].prefix;
    return ((m < lo ? lo : (m > hi ? hi : m)) << 32) | 0x80000000ull;
}

// Sum of squares of block s of a tensor tiled exactly by its 2-D blocks, added in row-major order.
__device__ inline double block_sumsq(const TensorDesc& td, u32 s) {
    const u32 d3 = td.d[3], b2 = td.b[2], b3 = td.b[3];
    const u32 G3 = fast_div(d3, td.fd[kDivB3]);
    const u32 g2 = s / G3, g3 = s - g2 * G3;
    const float* p = td.w + static_cast<u64>(g2) * b2 * d3 + static_cast<u64>(g3) * b3;
    double acc = 0.0;
    for (u32 r = 0; r < b2; ++r)
        for (u32 x = 0; x < b3; x += 4) acc = add_squares(acc, *reinterpret_cast<const float4*>(p + static_cast<u64>(r) * d3 + x));
    return acc;
}

// The sample and the level-0 histogram of its keys.  Four neighbouring blocks are taken per stride of four
// (jittered): their rows share 128-byte lines, so the sample costs a third of what single blocks at four times
// as many places cost, and the window's margin already counts a unit of four neighbours as one draw.
__global__ __launch_bounds__(kSampleHistThreads) void k_struct_sample_hist(StructArgs a, StructWindowArgs w, ArrayArgs ar) {
    __shared__ u32 s_hist[kBins];
    const int tid = threadIdx.x;
    const Level L0 = level_of(31, 0);
    for (int i = tid; i < kBins; i += kSampleHistThreads) s_hist[i] = 0;
    __syncthreads();
    for (u64 u = static_cast<u64>(blockIdx.x) * kSampleHistThreads + tid; u < w.n_units; u += static_cast<u64>(gridDim.x) * kSampleHistThreads) {
        const u64 q = u >> 2;
        const u64 jitter = (w.stride > 1) ? static_cast<u64>(mix32(static_cast<u32>(q) ^ static_cast<u32>(q >> 32))) % w.stride : 0;
        const u64 id = (q * w.stride + jitter) * 4 + (u & 3);
        u32 key = kNoKey;
        if (id < a.F) {
            const int t = tensor_of_struct_guess(a.td, a.n_tensors, a.F, id);
            const TensorDesc& td = a.td[t];
            const double acc = block_sumsq(td, static_cast<u32>(id - td.struct_start));
            key = static_cast<u32>((static_cast<u64>(__double_as_longlong(acc)) & 0x7FFFFFFFFFFFFFFFull) >> 32);
            atomicAdd(&s_hist[key >> L0.shift], 1u);
        }
        w.sample[u] = key;
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

// 8x8 blocks, every matrix a whole number of 64-block runs wide (so the 64 blocks of a wavefront lie in one
// block row of one tensor), rows 16-byte aligned.  Loads and lane layout as in k_struct_sumsq_tiles<2>:
// lane l fetches the l-th and the (64 + l)-th float4 of the run of every matrix row, even lanes own the
// run's blocks 0..31 and odd lanes blocks 32..63, neighbouring lanes trade the halves they fetched for each
// other, and the squares are added in row-major order.  The fetched values stay in registers; every lane
// then writes theta and mask for the two float4 it fetched, with the decision of the block each belongs to.
template <int THREADS>
__global__ __launch_bounds__(THREADS) void k_struct_tiles_fused(StructArgs a, StructWindowArgs w, double* sumsq, float* norms) {
    const u32 lane = threadIdx.x & 63u;
    const u64 wb = static_cast<u64>(blockIdx.x) * THREADS + (threadIdx.x & ~63u);   // the wavefront's first block
    if (wb >= a.F) return;
    const int t = tensor_of_struct_guess(a.td, a.n_tensors, a.F, wb);
    const TensorDesc& td = a.td[t];
    const u32 d3 = td.d[3];
    const u32 G3 = fast_div(d3, td.fd[kDivB3]);
    const u32 s0 = static_cast<u32>(wb - td.struct_start);
    const u32 g2 = s0 / G3, g3 = s0 - g2 * G3;
    const u64 e0 = static_cast<u64>(g2) * 8u * d3 + static_cast<u64>(g3) * 8u + lane * 4u;   // this lane's first float4
    const float* p = td.w + e0;
    const u32 half = lane & 1u;
    const u64 u = wb + (lane >> 1) + (half ? 32u : 0u);
    float4 va[8], vb[8];
#pragma unroll
    for (int r = 0; r < 8; ++r) {
        va[r] = ld4_stream(p + static_cast<u64>(r) * d3);
        vb[r] = ld4_stream(p + static_cast<u64>(r) * d3 + 256);
    }
    const u64 lo = window_lo63(w.wslots), hi = window_hi63(w.wslots), mid = window_mid63(w.wslots);
    double acc = 0.0;
#pragma unroll
    for (int r = 0; r < 8; ++r) {
        const float4 send = half ? va[r] : vb[r];
        float4 recv;
        recv.x = __shfl_xor(send.x, 1); recv.y = __shfl_xor(send.y, 1);
        recv.z = __shfl_xor(send.z, 1); recv.w = __shfl_xor(send.w, 1);
        acc = add_squares(acc, half ? recv : va[r]);
        acc = add_squares(acc, half ? vb[r] : recv);
    }
    const u64 key = static_cast<u64>(__double_as_longlong(acc)) & 0x7FFFFFFFFFFFFFFFull;
    a.keys[u] = key;
    if (sumsq) sumsq[u] = acc;
    if (norms) norms[u] = static_cast<float>(sqrt(acc));
    const bool keep = key > mid;                           // final outside the window, provisional inside
    const bool listed = key >= lo && key <= hi;
    a.smask[u] = keep ? 1 : 0;                             // the structure mask starts from the same decision
    // the first float4 a lane fetched belongs to the block of the even lane of its pair, the second to the odd one's
    const u64 kb = __ballot(keep);
    const bool keep_a = (kb >> (lane & ~1u)) & 1ull, keep_b = (kb >> (lane | 1u)) & 1ull;
    const OutDesc o = w.out[t];
    if (o.theta) {
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            float* q = o.theta + e0 + static_cast<u64>(r) * d3;
            st4_stream(q, keep_a ? va[r].x : 0.0f, keep_a ? va[r].y : 0.0f, keep_a ? va[r].z : 0.0f, keep_a ? va[r].w : 0.0f);
            st4_stream(q + 256, keep_b ? vb[r].x : 0.0f, keep_b ? vb[r].y : 0.0f, keep_b ? vb[r].z : 0.0f, keep_b ? vb[r].w : 0.0f);
        }
    }
    if (o.mask) {
        const u8 ma = keep_a ? 1 : 0, mb = keep_b ? 1 : 0;
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            u8* q = o.mask + e0 + static_cast<u64>(r) * d3;
            st_mask4_stream(q, ma, ma, ma, ma);
            st_mask4_stream(q + 256, mb, mb, mb, mb);
        }
    }
    // counts and list, one reservation per wavefront on the segment chosen by the workgroup
    const u32 seg = blockIdx.x % w.n_segs;
    const u32 n_above = static_cast<u32>(__popcll(__ballot(key > hi)));
    if (lane == 0 && n_above)
        atomicAdd(reinterpret_cast<unsigned long long*>(&w.seg_above[seg]), static_cast<unsigned long long>(n_above));
    const u64 lb = __ballot(listed);
    if (lb == 0) return;
    const int leader = __ffsll(static_cast<long long>(lb)) - 1;
    u64 b = 0;
    if (static_cast<int>(lane) == leader)
        b = atomicAdd(reinterpret_cast<unsigned long long*>(&w.seg_cnt[seg]), static_cast<unsigned long long>(__popcll(lb)));
    const u32 blo = __shfl(static_cast<u32>(b), leader, 64), bhi = __shfl(static_cast<u32>(b >> 32), leader, 64);
    if (listed) {
        const u64 pos = ((static_cast<u64>(bhi) << 32) | blo) + __popcll(lb & ((static_cast<u64>(1) << lane) - 1));
        if (pos < w.seg_cap) {
            w.cand_id[static_cast<u64>(seg) * w.seg_cap + pos] = static_cast<u32>(u);
            w.cand_key[static_cast<u64>(seg) * w.seg_cap + pos] = key;
        }
    }
}

// After the sweep: the rank to find among the listed blocks, or failure (the threshold lies outside the window,
// or the list overflowed), which leaves the ranking as the host armed it, for the levels over all aggregates.
__global__ __launch_bounds__(kBlock) void k_struct_window_check(StructArgs a, StructWindowArgs w) {
    __shared__ u64 s_wave[kBlock / 64];
    __shared__ u32 s_over;
    const int tid = threadIdx.x;
    if (tid == 0) s_over = 0;
    __syncthreads();
    u64 cnt = 0, abv = 0;
    bool over = false;
    for (u32 seg = tid; seg < w.n_segs; seg += kBlock) {
        const u64 c = w.seg_cnt[seg];
        over = over || (c > w.seg_cap);
        cnt += c;
        abv += w.seg_above[seg];
    }
    if (over) s_over = 1;
    u64 listed, above;
    block_excl_scan_u64(cnt, s_wave, &listed);
    block_excl_scan_u64(abv, s_wave, &above);
    __syncthreads();
    if (tid != 0) return;
    Slot& s = a.slots[0];
    if (s.state != kSelecting) return;
    if (s_over || above >= s.k || s.k - above > listed) {
        s.path = 3;                                        // reported: the window did not resolve this ranking
        atomicOr(&a.ctl->window_failed, 1u);
        return;
    }
    const u64 lo = window_lo63(w.wslots), hi = window_hi63(w.wslots);
    s.remaining = s.k - above;
    s.lo = lo;
    s.hi = hi;
    // leading digits shared by lo and hi are shared by every listed block: those levels need no counting
    u32 begin = 0;
    u64 prefix = 0;
    const int nl = n_levels(63);
    for (int level = 0; level < nl - 1; ++level) {
        const Level L = level_of(63, level);
        if (((lo ^ hi) >> L.shift) != 0) break;
        prefix = (lo >> L.shift) << L.shift;
        begin = level + 1;
    }
    s.prefix = prefix;
    s.level_begin = begin;
}

// Histogram of one radix level over the listed blocks' keys; the level before it is folded in first, as in
// k_hist_keys.  Few wide workgroups, each taking four of the short segments at a time.
__global__ __launch_bounds__(kArrayThreads) void k_hist_listed_keys(StructArgs a, StructWindowArgs w, int level) {
    __shared__ u32 s_hist[kBins];
    __shared__ u64 s_prefix;
    __shared__ u32 s_active;
    if (a.ctl->window_failed != 0) return;                 // the levels over all aggregates run instead
    const int tid = threadIdx.x;
    if (tid < 64) {
        const SlotStep e = (level == 0) ? slot_canonical(a.slots[0])
                                        : wave_enter_level(a.slots[0], level, 63, struct_hist(a, level - 1), struct_coarse(a, level - 1));
        if (tid == 0) {
            s_prefix = e.prefix;
            s_active = (e.state == kSelecting && static_cast<u32>(level) >= a.slots[0].level_begin) ? 1u : 0u;
            if (blockIdx.x == 0 && level > 0) a.slots[0].step[level & 1] = e;
        }
    }
    for (int i = tid; i < kBins; i += kArrayThreads) s_hist[i] = 0;
    __syncthreads();
    if (!s_active) return;                                 // uniform: a level that lo and hi share, or nothing to rank
    const Level L = level_of(63, level);
    const int nb = 1 << L.bits;
    const u64 prefix = s_prefix;
    constexpr int kSegBatch = 4, kPer = 2;
    for (u32 seg0 = blockIdx.x; seg0 < w.n_segs; seg0 += gridDim.x * kSegBatch) {
        u64 cnt[kSegBatch], first[kSegBatch], most = 0;
#pragma unroll
        for (int b = 0; b < kSegBatch; ++b) {
            const u64 seg = static_cast<u64>(seg0) + static_cast<u64>(b) * gridDim.x;
            u64 c = (seg < w.n_segs) ? w.seg_cnt[seg] : 0;
            if (c > w.seg_cap) c = w.seg_cap;
            cnt[b] = c;
            first[b] = seg * w.seg_cap;
            most = c > most ? c : most;
        }
        for (u64 i0 = tid; i0 < most; i0 += static_cast<u64>(kArrayThreads) * kPer) {
            u64 key[kSegBatch * kPer];
#pragma unroll
            for (int u = 0; u < kSegBatch * kPer; ++u) {
                const u64 i = i0 + static_cast<u64>(kArrayThreads) * (u / kSegBatch);
                key[u] = (i < cnt[u % kSegBatch]) ? w.cand_key[first[u % kSegBatch] + i] : ~prefix;   // a filler that fails the prefix test
            }
#pragma unroll
            for (int u = 0; u < kSegBatch * kPer; ++u)
                if (i0 + static_cast<u64>(kArrayThreads) * (u / kSegBatch) < cnt[u % kSegBatch] && ((key[u] ^ prefix) >> L.hi_shift) == 0)
                    atomicAdd(&s_hist[(key[u] >> L.shift) & (nb - 1)], 1u);
        }
    }
    __syncthreads();
    u64* dst = struct_hist(a, level);
    for (int i = tid; i < nb; i += kArrayThreads) {
        const u32 v = s_hist[i];
        if (v) atomicAdd(reinterpret_cast<unsigned long long*>(dst + i), static_cast<unsigned long long>(v));
    }
    if (tid < kCoarse) {
        const int run = coarse_run(nb);
        u32 v = 0;
        for (int t = tid * run; t < (tid + 1) * run && t < nb; ++t) v += s_hist[t];
        if (v) atomicAdd(reinterpret_cast<unsigned long long*>(struct_coarse(a, level) + tid), static_cast<unsigned long long>(v));
    }
}

// Rewrites the listed blocks whose final decision differs from the provisional one (one thread per block).
__global__ __launch_bounds__(kBlock) void k_struct_fixup(StructArgs a, StructWindowArgs w) {
    if (a.ctl->window_failed != 0) return;                 // the gated apply sweep rewrites everything
    const Slot& s = a.slots[0];
    const u64 T = s.prefix, tie_end = s.tie_end;
    const u64 mid = window_mid63(w.wslots);
    const u32 parts = gridDim.x / w.n_segs;
    const u32 seg = blockIdx.x % w.n_segs, part = blockIdx.x / w.n_segs;
    if (part >= parts) return;
    u64 cnt = w.seg_cnt[seg];
    if (cnt > w.seg_cap) cnt = w.seg_cap;
    for (u64 i = static_cast<u64>(part) * kBlock + threadIdx.x; i < cnt; i += static_cast<u64>(parts) * kBlock) {
        const u64 id = w.cand_id[static_cast<u64>(seg) * w.seg_cap + i];
        const u64 key = w.cand_key[static_cast<u64>(seg) * w.seg_cap + i];
        const bool was_kept = key > mid;
        const bool keep = key > T || (key == T && id < tie_end);
        if (keep == was_kept) continue;
        a.smask[id] = keep ? 1 : 0;
        const int t = tensor_of_struct_guess(a.td, a.n_tensors, a.F, id);
        const TensorDesc& td = a.td[t];
        const u32 d3 = td.d[3];
        const u32 G3 = fast_div(d3, td.fd[kDivB3]);
        const u32 sidx = static_cast<u32>(id - td.struct_start);
        const u32 g2 = sidx / G3, g3 = sidx - g2 * G3;
        const u64 e0 = static_cast<u64>(g2) * 8u * d3 + static_cast<u64>(g3) * 8u;
        const OutDesc o = w.out[t];
        const u32 m4 = keep ? 0x01010101u : 0u;
        for (u32 r = 0; r < 8; ++r) {
            const u64 e = e0 + static_cast<u64>(r) * d3;
            if (o.theta) {
                float4 x0 = make_float4(0.f, 0.f, 0.f, 0.f), x1 = x0;
                if (keep) {
                    x0 = *reinterpret_cast<const float4*>(td.w + e);
                    x1 = *reinterpret_cast<const float4*>(td.w + e + 4);
                }
                *reinterpret_cast<float4*>(o.theta + e) = x0;
                *reinterpret_cast<float4*>(o.theta + e + 4) = x1;
            }
            if (o.mask) {
                *reinterpret_cast<u32*>(o.mask + e) = m4;
                *reinterpret_cast<u32*>(o.mask + e + 4) = m4;
            }
        }
    }
}

// Full apply sweep that runs only when the window failed: a fixed, modest grid walks the tiles.
template <bool VEC>
__global__ __launch_bounds__(kBlock) void k_struct_apply_gated(StructArgs a, const OutDesc* __restrict__ out, u64 n_tiles) {
    if (a.ctl->window_failed == 0) return;
    for (u64 tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) struct_apply_tile<VEC>(a, out, tile);
}

}  // namespace condensa
