// Streaming mask/apply kernels: theta = keep ? x : +0 with optional fp16 rounding (Prune and
// Compose([Prune, Quantize]), Table 1) and the fused L-C multiplier / penalty-gradient update
// (Section 3.3).  128-bit accesses when every pointer is aligned.
#pragma once
#include "k_select.h"

namespace condensa {

// The apply sweeps run one workgroup per 1024 elements (one float4 per thread): many short
// workgroups keep more independent HBM streams in flight than long ones.
constexpr int kSubPerChunk = kChunk / (kBlock * 4);     // 8 workgroups share a chunk

// keep rule of the selection: key above the threshold, or equal to it with index below tie_end
__device__ inline bool keep_rule(u32 key, u32 T, u64 idx, u64 tie_end) {
    return key > T || (key == T && idx < tie_end);
}

// Workgroups that lie wholly inside their tensor (all but a tensor's last) take the unguarded 128-bit
// accesses; the selection record and the output table are read before the data so that their latency
// overlaps the data loads.
template <bool VEC>
__device__ inline void prune_apply_tile(const DataArgs& a, const OutDesc* __restrict__ out, u64 tile) {
    __shared__ u32 s_T[kMaxJ];
    __shared__ u64 s_end[kMaxJ];
    __shared__ OutDesc s_out[kMaxJ];
    const u64 c = tile / kSubPerChunk;
    const u32 sub = static_cast<u32>(tile % kSubPerChunk);
    if (c >= a.n_chunks) return;
    const int tid = threadIdx.x;
    const int t = static_cast<int>(a.chunk_map[c]);
    const u64 g = a.per_tensor ? t : 0;
    const TensorDesc& td = a.td[t];
    const u64 n = td.n;
    const u64 wg0 = (c - td.chunk_start) * kChunk + static_cast<u64>(sub) * (kBlock * 4);
    if (wg0 >= n) return;                                                // uniform
    if (tid < a.J) {
        const Slot& s = a.slots[g * a.J + tid];
        s_T[tid] = static_cast<u32>(s.prefix);
        s_end[tid] = s.tie_end;
        s_out[tid] = out[static_cast<u64>(tid) * a.n_tensors + t];
    }
    const u64 idx0 = a.per_tensor ? 0 : td.flat_start;
    const u64 e0 = wg0 + tid * 4;
    const bool full = VEC && wg0 + kBlock * 4 <= n;                      // uniform
    float v[4] = {0.f, 0.f, 0.f, 0.f};
    if (full) {
        const float4 x = ld4_stream(td.w + e0);
        v[0] = x.x; v[1] = x.y; v[2] = x.z; v[3] = x.w;
    } else if (e0 < n) {
        load4<VEC>(td.w, e0, n, v);
    }
    __syncthreads();
    if (e0 >= n) return;
    u32 key[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) key[k] = mag_key(v[k]);
    for (int j = 0; j < a.J; ++j) {
        const u32 T = s_T[j];
        const u64 end = s_end[j];
        float th[4];
        u8 m[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const bool keep = keep_rule(key[k], T, idx0 + e0 + k, end);
            m[k] = keep ? 1 : 0;
            th[k] = keep ? v[k] : 0.0f;
        }
        const OutDesc& o = s_out[j];
        if (full) {
            if (o.theta) st4_stream(o.theta + e0, th[0], th[1], th[2], th[3]);
            if (o.theta16) {
                st_code4_stream(o.theta16 + e0, f32_to_f16_rne(th[0]), f32_to_f16_rne(th[1]), f32_to_f16_rne(th[2]), f32_to_f16_rne(th[3]));
            }
            if (o.mask) st_mask4_stream(o.mask + e0, m[0], m[1], m[2], m[3]);
        } else {
            if (o.theta) store4<VEC>(o.theta, e0, n, th);
            if (o.theta16) {
                u16 h[4];
#pragma unroll
                for (int k = 0; k < 4; ++k) h[k] = f32_to_f16_rne(th[k]);
                store4_u16<VEC>(o.theta16, e0, n, h);
            }
            if (o.mask) store4_u8<VEC>(o.mask, e0, n, m);
        }
    }
}

template <bool VEC>
__global__ __launch_bounds__(kBlock) void k_prune_apply(DataArgs a, const OutDesc* __restrict__ out) {
    prune_apply_tile<VEC>(a, out, blockIdx.x);
}

// theta = C(w - lambda/mu) entries, lambda' = lambda - mu (w - theta), g = mu (w - theta) - lambda',
// each operation rounded once in binary32.  THREADS threads per workgroup, one float4 each.
// PQ: the composed scheme Compose([Prune(), Quantize(float16)]) -- theta is rounded to binary16 and the
// update sees its exact widening D(theta).  One float4 per thread in 64-thread workgroups measured best
// for this 2-read 3-write kernel (more per thread or wider workgroups lose 10-15%).
template <bool PQ>
__device__ inline void lc_update4(const float w[4], const float l[4], float mu, u32 T, u64 idx, u64 end,
                                  float th[4], float ln[4], float gr[4], u8 m[4], u16 h[4]) {
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const float v = lc_shift(w[k], l[k], mu);
        const bool keep = keep_rule(mag_key(v), T, idx + k, end);
        m[k] = keep ? 1 : 0;
        th[k] = keep ? v : 0.0f;
        h[k] = 0;
        if (PQ) {
            h[k] = f32_to_f16_rne(th[k]);
            th[k] = f16_bits_to_f32(h[k]);
        }
        const float e = __fsub_rn(w[k], th[k]);
        const float p = __fmul_rn(mu, e);
        ln[k] = __fsub_rn(l[k], p);
        gr[k] = __fsub_rn(p, ln[k]);
    }
}

template <bool VEC, int THREADS, bool PQ, int QUADS>
__device__ inline void lc_apply_tile(const DataArgs& a, const OutDesc* __restrict__ out, u64 tile) {
    constexpr u32 kTile = THREADS * 4 * QUADS;
    constexpr u32 kSub = kChunk / kTile;
    const u64 c = tile / kSub;
    const u32 sub = static_cast<u32>(tile % kSub);
    if (c >= a.n_chunks) return;
    const int tid = threadIdx.x;
    const int t = static_cast<int>(a.chunk_map[c]);
    const TensorDesc& td = a.td[t];
    const u64 n = td.n;
    const u64 wg0 = (c - td.chunk_start) * kChunk + static_cast<u64>(sub) * kTile;
    if (wg0 >= n) return;                                                // uniform
    const Slot& s = a.slots[0];
    const u32 T = static_cast<u32>(s.prefix);
    const u64 end = s.tie_end;
    const OutDesc o = out[t];
    const float mu = a.mu;
    u32 nz = 0;                                                          // PQ: stored codes other than +-0
    if (VEC && wg0 + kTile <= n) {                                       // uniform
        float4 x[QUADS], y[QUADS];
#pragma unroll
        for (int q = 0; q < QUADS; ++q) {
            x[q] = ld4_stream(td.w + wg0 + q * (THREADS * 4) + tid * 4);
            y[q] = ld4_stream(td.lam + wg0 + q * (THREADS * 4) + tid * 4);
        }
#pragma unroll
        for (int q = 0; q < QUADS; ++q) {
            const u64 e0 = wg0 + q * (THREADS * 4) + tid * 4;
            const float w[4] = {x[q].x, x[q].y, x[q].z, x[q].w};
            const float l[4] = {y[q].x, y[q].y, y[q].z, y[q].w};
            float th[4], ln[4], gr[4];
            u8 m[4];
            u16 h[4];
            lc_update4<PQ>(w, l, mu, T, td.flat_start + e0, end, th, ln, gr, m, h);
            if (PQ) nz += ((h[0] & 0x7FFFu) != 0) + ((h[1] & 0x7FFFu) != 0) + ((h[2] & 0x7FFFu) != 0) + ((h[3] & 0x7FFFu) != 0);
            if (o.theta) st4_stream(o.theta + e0, th[0], th[1], th[2], th[3]);
            if (PQ && o.theta16) {
                st_code4_stream(o.theta16 + e0, h[0], h[1], h[2], h[3]);
            }
            st4_stream(td.lam_out + e0, ln[0], ln[1], ln[2], ln[3]);
            if (td.grad) st4_stream(td.grad + e0, gr[0], gr[1], gr[2], gr[3]);
            if (o.mask) st_mask4_stream(o.mask + e0, m[0], m[1], m[2], m[3]);
        }
    } else {
        for (int q = 0; q < QUADS; ++q) {
            const u64 e0 = wg0 + q * (THREADS * 4) + tid * 4;
            if (e0 >= n) break;
            float w[4], l[4], th[4], ln[4], gr[4];
            u8 m[4];
            u16 h[4];
            load4<VEC>(td.w, e0, n, w);
            load4<VEC>(td.lam, e0, n, l);
            lc_update4<PQ>(w, l, mu, T, td.flat_start + e0, end, th, ln, gr, m, h);
            if (PQ) for (int k = 0; k < 4; ++k) nz += (e0 + k < n) && (h[k] & 0x7FFFu) != 0;
            if (o.theta) store4<VEC>(o.theta, e0, n, th);
            if (PQ && o.theta16) store4_u16<VEC>(o.theta16, e0, n, h);
            store4<VEC>(td.lam_out, e0, n, ln);
            if (td.grad) store4<VEC>(td.grad, e0, n, gr);
            if (o.mask) store4_u8<VEC>(o.mask, e0, n, m);
        }
    }
    if (PQ && a.nnz_seg) {                                               // one atomic per wavefront, spread over the segments
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) nz += __shfl_down(nz, d, 64);
        if ((tid & 63) == 0 && nz)
            atomicAdd(reinterpret_cast<unsigned long long*>(&a.nnz_seg[(tile * (THREADS / 64) + (tid >> 6)) % kNnzSegs]), static_cast<unsigned long long>(nz));
    }
}

// Footprint objective of the prune + binary16 L-C step (Evaluation, Objective 1): the number of stored codes
// other than +-0, from the counters that the sweeps left.  One-sweep form that held: the sweep's own count
// (upper halves of the `above` counters) corrected by the fix-up pass; otherwise the apply sweep's count.
__global__ __launch_bounds__(kBlock) void k_nnz_finish(DataArgs a, const u64* __restrict__ seg_above, int one_sweep, u64* nnz_out) {
    __shared__ u64 s_wave[kBlock / 64];
    const bool sweep = one_sweep && a.ctl->window_failed == 0;
    u64 v = 0;
    for (int i = threadIdx.x; i < kNnzSegs; i += kBlock) v += sweep ? (seg_above[i] >> 32) : a.nnz_seg[i];
    u64 total;
    block_excl_scan_u64(v, s_wave, &total);
    if (threadIdx.x == 0) *nnz_out = sweep ? total + a.ctl->nnz_delta : total;
}

template <bool VEC, int THREADS, bool PQ, int QUADS = 1>
__global__ __launch_bounds__(THREADS) void k_lc_apply(DataArgs a, const OutDesc* __restrict__ out) {
    lc_apply_tile<VEC, THREADS, PQ, QUADS>(a, out, blockIdx.x);
}

// ---- learning-step update with the penalty gradient folded in -----------------------------------------
// g = grad L + mu (w - theta) - lambda;  buf' = m buf + g;  w' = w - lr buf'   (binary32, one rounding per
// operation).  Table roles: td.w = weights (updated in place), td.grad = grad L, td.lam = lambda,
// td.lam_out = momentum buffer (updated in place), out[t].theta = theta.
template <bool VEC>
__global__ __launch_bounds__(64) void k_lc_sgd(DataArgs a, const OutDesc* __restrict__ out, float lr, float momentum) {
    constexpr u32 kSub = kChunk / 256;
    const u64 c = blockIdx.x / kSub;
    const u32 sub = blockIdx.x % kSub;
    if (c >= a.n_chunks) return;
    const int t = static_cast<int>(a.chunk_map[c]);
    const TensorDesc& td = a.td[t];
    const u64 n = td.n;
    const u64 wg0 = (c - td.chunk_start) * kChunk + static_cast<u64>(sub) * 256;
    if (wg0 >= n) return;                                                // uniform
    const u64 e0 = wg0 + threadIdx.x * 4;
    const float* theta = out[t].theta;
    const bool full = VEC && wg0 + 256 <= n;                             // uniform
    float w[4], g[4], th[4], l[4], b[4];
    if (full) {
        const float4 x0 = ld4_stream(td.w + e0), x1 = ld4_stream(td.grad + e0), x2 = ld4_stream(theta + e0),
                     x3 = ld4_stream(td.lam + e0), x4 = ld4_stream(td.lam_out + e0);
        w[0] = x0.x; w[1] = x0.y; w[2] = x0.z; w[3] = x0.w;
        g[0] = x1.x; g[1] = x1.y; g[2] = x1.z; g[3] = x1.w;
        th[0] = x2.x; th[1] = x2.y; th[2] = x2.z; th[3] = x2.w;
        l[0] = x3.x; l[1] = x3.y; l[2] = x3.z; l[3] = x3.w;
        b[0] = x4.x; b[1] = x4.y; b[2] = x4.z; b[3] = x4.w;
    } else {
        if (e0 >= n) return;
        load4<VEC>(td.w, e0, n, w);
        load4<VEC>(td.grad, e0, n, g);
        load4<VEC>(theta, e0, n, th);
        load4<VEC>(td.lam, e0, n, l);
        load4<VEC>(td.lam_out, e0, n, b);
    }
    float wn[4], bn[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const float t1 = __fsub_rn(w[k], th[k]);
        const float t2 = __fmul_rn(a.mu, t1);
        const float t3 = __fadd_rn(g[k], t2);
        const float t4 = __fsub_rn(t3, l[k]);
        const float t5 = __fmul_rn(momentum, b[k]);
        bn[k] = __fadd_rn(t5, t4);
        wn[k] = __fsub_rn(w[k], __fmul_rn(lr, bn[k]));
    }
    if (full) {
        st4_stream(td.lam_out + e0, bn[0], bn[1], bn[2], bn[3]);
        st4_stream(const_cast<float*>(td.w) + e0, wn[0], wn[1], wn[2], wn[3]);
    } else {
        store4<VEC>(td.lam_out, e0, n, bn);
        store4<VEC>(const_cast<float*>(td.w), e0, n, wn);
    }
}

// ---- footprint objective: number of non-zero parameters (Evaluation, Objective 1) ---------------------
// Persistent workgroups, one chunk per step; the loads of the next chunk are requested before the current
// one is counted.  Per-workgroup counts go to `partial`; k_sum_partials adds them up, so the result needs
// no atomics and no cleared memory.
// KIND: 0 = binary32 values, 1 = 16-bit floating-point codes, 2 = 8-bit floating-point codes (a chunk
// is kChunk elements of that width); a zero is a code whose bits below the sign are all clear.
template <int KIND, bool VEC>
__global__ __launch_bounds__(kBlock) void k_count_nonzero(DataArgs a, u64* partial) {
    __shared__ u64 s_wave[kBlock / 64];
    constexpr int R = kQuadsPerThread >> KIND;              // 128-bit loads per thread and chunk: 8, 4, 2
    const int tid = threadIdx.x;
    u64 cnt = 0;
    f32x4 nxt[R];
    bool nxt_full = false;
    // requests chunk c's data when the whole chunk lies inside its tensor (the same for every thread)
    auto request = [&](u64 c) {
        nxt_full = false;
        if (!VEC || c >= a.n_chunks) return;
        const TensorDesc& td = a.td[a.chunk_map[c]];
        const u64 base = (c - td.chunk_start) * kChunk;
        if (base + kChunk > td.n) return;
        nxt_full = true;
        const char* p = reinterpret_cast<const char*>(td.w) + (base << (2 - KIND));      // 4, 2 or 1 byte per element
#pragma unroll
        for (int q = 0; q < R; ++q)
            nxt[q] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p) + q * kBlock + tid);
    };
    request(blockIdx.x);
    for (u64 c = blockIdx.x; c < a.n_chunks; c += gridDim.x) {
        f32x4 cur[R];
#pragma unroll
        for (int q = 0; q < R; ++q) cur[q] = nxt[q];
        const bool full = nxt_full;
        request(c + gridDim.x);
        if (full) {
#pragma unroll
            for (int q = 0; q < R; ++q)
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const u32 bits = __float_as_uint(cur[q][k]);
                    if (KIND == 0) cnt += (bits & 0x7FFFFFFFu) != 0;
                    if (KIND == 1) cnt += ((bits & 0x7FFFu) != 0) + ((bits & 0x7FFF0000u) != 0);
                    if (KIND == 2) cnt += ((bits & 0x7Fu) != 0) + ((bits & 0x7F00u) != 0) + ((bits & 0x7F0000u) != 0) +
                                          ((bits & 0x7F000000u) != 0);
                }
            continue;
        }
        const TensorDesc& td = a.td[a.chunk_map[c]];
        const u64 base = (c - td.chunk_start) * kChunk;
        for (int q = 0; q < kQuadsPerThread; ++q) {
            const u64 e0 = base + static_cast<u64>(q) * (kBlock * 4) + tid * 4;
            if (e0 >= td.n) break;
            if (KIND == 2) {
                const u8* p = reinterpret_cast<const u8*>(td.w);
                for (int k = 0; k < 4; ++k) if (e0 + k < td.n) cnt += (p[e0 + k] & 0x7Fu) != 0;
            } else if (KIND == 1) {
                const u16* p = reinterpret_cast<const u16*>(td.w);
                if (VEC && e0 + 4 <= td.n) {
                    const ushort4 v = *reinterpret_cast<const ushort4*>(p + e0);
                    cnt += ((v.x & 0x7FFFu) != 0) + ((v.y & 0x7FFFu) != 0) + ((v.z & 0x7FFFu) != 0) + ((v.w & 0x7FFFu) != 0);
                } else {
                    for (int k = 0; k < 4; ++k) if (e0 + k < td.n) cnt += (p[e0 + k] & 0x7FFFu) != 0;
                }
            } else {
                float v[4];
                load4<VEC>(td.w, e0, td.n, v);      // missing elements read as 0
#pragma unroll
                for (int k = 0; k < 4; ++k) cnt += mag_key(v[k]) != 0;
            }
        }
    }
    u64 total;
    block_excl_scan_u64(cnt, s_wave, &total);
    if (tid == 0) partial[blockIdx.x] = total;
}

__global__ __launch_bounds__(kBlock) void k_sum_partials(const u64* partial, u32 n, u64* out) {
    __shared__ u64 s_wave[kBlock / 64];
    u64 v = 0;
    for (u32 i = threadIdx.x; i < n; i += kBlock) v += partial[i];
    u64 total;
    block_excl_scan_u64(v, s_wave, &total);
    if (threadIdx.x == 0) *out = total;
}

}  // namespace condensa
