// One density on the sampled-window path: selection sweep and apply sweep in one pass.
//
// The window [lo, hi] is known before the sweep, and unless the sample was unlucky the threshold lies
// inside it.  So the sweep can already write the final outputs of every element outside the window --
// kept above hi, dropped below lo -- and a provisional decision for the few elements inside it: kept iff
// the key exceeds `mid`, the sample's own estimate of the threshold.  It stores the inputs of those
// elements with the candidates.  Once the threshold and the tie rule are resolved on the candidate list,
// a fix-up pass rewrites the candidates whose final decision differs from the provisional one (the keys
// between the estimate and the threshold: a few percent of the candidates; scattered 4-byte writes are
// slow on this memory system, about 6 G/s, so their number matters).
// The weights (and multipliers) are then read once instead of twice: 9 instead of 13 bytes per weight
// for theta + mask, 20 instead of 28 for the L-C step (Section 3.3).  If the window turns out not to
// hold the threshold, the radix levels find it and a full apply sweep, gated on that failure, rewrites
// every output; that is why the inputs must not be overwritten (no in-place theta or lambda here).
#pragma once
#include "k_apply.h"
#include "k_window.h"

namespace condensa {

// The provisional threshold: the ranked sample key, forced into the window (a failed ranking leaves an
// arbitrary value; any value inside the window is valid, both kernels only have to agree on it).
__device__ inline u32 window_mid(u32 ranked, u32 lo, u32 hi) {
    return ranked < lo ? lo : (ranked > hi ? hi : ranked);
}

// PQ (with LC): theta is rounded to binary16 and the update sees its exact widening, as in k_lc_apply.
template <bool LC, bool VEC, int QUADS, bool PQ>
__global__ __launch_bounds__(64) void k_window_fused(DataArgs a, WindowArgs w) {
    constexpr int kWaveElems = 256 * QUADS;
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
    const u32 hi = static_cast<u32>(w.wslots[0].prefix);
    const u32 lo = static_cast<u32>(w.wslots[1].prefix);
    const u32 span = hi - lo;
    const u32 mid = window_mid(static_cast<u32>(w.wslots[2].prefix), lo, hi);
    const OutDesc o = w.out[t];
    const float mu = a.mu;
    const bool full = VEC && base + kWaveElems <= n;                    // uniform over the wavefront

    float wk[QUADS][4], lk[QUADS][4];
    if (full) {
#pragma unroll
        for (int q = 0; q < QUADS; ++q) {
            const float4 x = ld4_stream(td.w + base + q * 256 + lane * 4);
            wk[q][0] = x.x; wk[q][1] = x.y; wk[q][2] = x.z; wk[q][3] = x.w;
            if (LC) {
                const float4 y = ld4_stream(td.lam + base + q * 256 + lane * 4);
                lk[q][0] = y.x; lk[q][1] = y.y; lk[q][2] = y.z; lk[q][3] = y.w;
            }
        }
    }
    u32 key[QUADS][4];
    u32 cmask = 0, above = 0, nz = 0;                                   // nz (PQ): stored codes other than +-0
#pragma unroll
    for (int q = 0; q < QUADS; ++q) {
        const u64 e0 = base + static_cast<u64>(q) * 256 + lane * 4;
        if (!full) {
#pragma unroll
            for (int k = 0; k < 4; ++k) { wk[q][k] = 0.0f; lk[q][k] = 0.0f; }
            if (e0 < n) {
                load4<VEC>(td.w, e0, n, wk[q]);
                if (LC) load4<VEC>(td.lam, e0, n, lk[q]);
            }
        }
        float th[4], ln[4], gr[4];
        u8 m[4];
        u16 h16[4] = {0, 0, 0, 0};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const float v = LC ? lc_shift(wk[q][k], lk[q][k], mu) : wk[q][k];
            const u32 x = mag_key(v);
            key[q][k] = x;
            const bool keep = x > mid;                                  // final outside the window, provisional inside
            if (full || e0 + k < n) {
                above += (x > hi) ? 1u : 0u;
                if (x - lo <= span) cmask |= 1u << (q * 4 + k);
            }
            m[k] = keep ? 1 : 0;
            th[k] = keep ? v : 0.0f;
            if (PQ) {
                h16[k] = f32_to_f16_rne(th[k]);
                th[k] = f16_bits_to_f32(h16[k]);
                nz += ((full || e0 + k < n) && (h16[k] & 0x7FFFu) != 0) ? 1u : 0u;
            }
            if (LC) {
                const float e = __fsub_rn(wk[q][k], th[k]);
                const float p = __fmul_rn(mu, e);
                ln[k] = __fsub_rn(lk[q][k], p);
                gr[k] = __fsub_rn(p, ln[k]);
            }
        }
        if (full) {
            if (o.theta) st4_stream(o.theta + e0, th[0], th[1], th[2], th[3]);
            if (!LC && o.theta16) {
                st_code4_stream(o.theta16 + e0, f32_to_f16_rne(th[0]), f32_to_f16_rne(th[1]), f32_to_f16_rne(th[2]), f32_to_f16_rne(th[3]));
            }
            if (PQ && o.theta16) {
                st_code4_stream(o.theta16 + e0, h16[0], h16[1], h16[2], h16[3]);
            }
            if (LC) {
                st4_stream(td.lam_out + e0, ln[0], ln[1], ln[2], ln[3]);
                if (td.grad) st4_stream(td.grad + e0, gr[0], gr[1], gr[2], gr[3]);
            }
            if (o.mask) st_mask4_stream(o.mask + e0, m[0], m[1], m[2], m[3]);
        } else if (e0 < n) {
            if (o.theta) store4<VEC>(o.theta, e0, n, th);
            if (!LC && o.theta16) {
                u16 h[4];
#pragma unroll
                for (int k = 0; k < 4; ++k) h[k] = f32_to_f16_rne(th[k]);
                store4_u16<VEC>(o.theta16, e0, n, h);
            }
            if (PQ && o.theta16) store4_u16<VEC>(o.theta16, e0, n, h16);
            if (LC) {
                store4<VEC>(td.lam_out, e0, n, ln);
                if (td.grad) store4<VEC>(td.grad, e0, n, gr);
            }
            if (o.mask) store4_u8<VEC>(o.mask, e0, n, m);
        }
    }
    // counts and candidates, as in k_window_sweep_wave; a candidate also keeps its inputs
    // (PQ: the non-zero count rides in the upper half of the same counter -- a segment holds fewer than 2^32 elements)
    const u32 seg = blockIdx.x % w.n_segs;
    u32 s = above;
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) s += __shfl_down(s, d, 64);
    u64 s64 = s;
    if (PQ) {
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) nz += __shfl_down(nz, d, 64);
        s64 |= static_cast<u64>(nz) << 32;
    }
    if (lane == 0 && s64)
        atomicAdd(reinterpret_cast<unsigned long long*>(&w.seg_region[seg]), static_cast<unsigned long long>(s64));
    const u32 cnt = __popc(cmask);
    u32 incl = cnt;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const u32 up = __shfl_up(incl, d, 64);
        if (lane >= d) incl += up;
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
                    w.cand_idx[first + pos] = cand_pack(td.flat_start + base + static_cast<u64>(q) * 256 + lane * 4 + k, t);
                    w.cand_w[first + pos] = wk[q][k];
                    if (LC) w.cand_lam[first + pos] = lk[q][k];
                }
                ++pos;
            }
        }
    }
}

constexpr unsigned kFixupParts = 4;   // workgroups per candidate segment in the fix-up pass (2, 4, 8 measure alike:
                                      // the pass is bound by its scattered 4-byte writes)

// Outputs of the candidates whose final decision differs from the provisional one of the fused sweep.
template <bool LC, bool PQ>
__global__ __launch_bounds__(kBlock) void k_window_fixup(DataArgs a, WindowArgs w) {
    if (a.ctl->window_failed != 0) return;                 // the gated apply sweep rewrites everything
    const Slot& s = a.slots[0];
    if (s.state != kDone) return;
    const u32 T = static_cast<u32>(s.prefix);
    const u64 tie_end = s.tie_end;
    const u32 mid = window_mid(static_cast<u32>(w.wslots[2].prefix), static_cast<u32>(s.lo), static_cast<u32>(s.hi));
    const float mu = a.mu;
    // `parts` workgroups share a segment (the per-candidate work is a chain of dependent loads, so the
    // kernel's time is set by how many candidates one thread walks through)
    const u32 parts = gridDim.x / w.n_segs;
    long long nz_delta = 0;                                // PQ: change of the count of non-zero codes
    {
        const u32 seg = blockIdx.x % w.n_segs, part = blockIdx.x / w.n_segs;
        if (part >= parts) return;
        u64 cnt = w.seg_cnt[seg];
        if (cnt > w.seg_cap) cnt = w.seg_cap;
        const u64 first = static_cast<u64>(seg) * w.seg_cap;
        for (u64 i = static_cast<u64>(part) * kBlock + threadIdx.x; i < cnt; i += static_cast<u64>(parts) * kBlock) {
            const u32 key = w.cand_key[first + i];
            const bool was_kept = key > mid;
            if (was_kept && key > T) continue;             // most candidates: decided without their index
            if (!was_kept && key < T) continue;
            const u64 packed = w.cand_idx[first + i];
            const u64 idx = cand_flat(packed);
            const bool keep = keep_rule(key, T, idx, tie_end);
            if (keep == was_kept) continue;
            const int t = cand_tensor(packed);
            const TensorDesc& td = a.td[t];
            const u64 e = idx - td.flat_start;
            const OutDesc o = w.out[t];
            const float wv = w.cand_w[first + i];
            if (LC) {
                const float lv = w.cand_lam[first + i];
                float th = keep ? lc_shift(wv, lv, mu) : 0.0f;
                if (PQ) {
                    const u16 h = f32_to_f16_rne(th);
                    th = f16_bits_to_f32(h);
                    if (o.theta16) o.theta16[e] = h;
                    // the sweep counted the code of the other decision: the kept value's code, or +0
                    const u16 hv = keep ? h : f32_to_f16_rne(lc_shift(wv, lv, mu));
                    if ((hv & 0x7FFFu) != 0) nz_delta += keep ? 1 : -1;
                }
                const float d = __fsub_rn(wv, th);
                const float p = __fmul_rn(mu, d);
                const float ln = __fsub_rn(lv, p);
                if (o.theta) o.theta[e] = th;
                td.lam_out[e] = ln;
                if (td.grad) td.grad[e] = __fsub_rn(p, ln);
            } else {
                const float th = keep ? wv : 0.0f;
                if (o.theta) o.theta[e] = th;
                if (o.theta16) o.theta16[e] = f32_to_f16_rne(th);
            }
            if (o.mask) o.mask[e] = keep ? 1 : 0;
        }
    }
    if (PQ && nz_delta != 0)
        atomicAdd(reinterpret_cast<unsigned long long*>(&a.ctl->nnz_delta), static_cast<unsigned long long>(nz_delta));
}

// Full apply sweeps that run only when the window failed: a fixed, modest grid walks the tiles, so that
// the usual case costs one empty launch.
template <bool VEC, bool PQ>
__global__ __launch_bounds__(64) void k_lc_apply_gated(DataArgs a, const OutDesc* __restrict__ out, u64 n_tiles) {
    if (a.ctl->window_failed == 0) return;
    for (u64 tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) lc_apply_tile<VEC, 64, PQ, 1>(a, out, tile);
}

template <bool VEC>
__global__ __launch_bounds__(kBlock) void k_prune_apply_gated(DataArgs a, const OutDesc* __restrict__ out, u64 n_tiles) {
    if (a.ctl->window_failed == 0) return;
    for (u64 tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        prune_apply_tile<VEC>(a, out, tile);
        __syncthreads();                                   // the tile's LDS tables are rewritten by the next one
    }
}

}  // namespace condensa
