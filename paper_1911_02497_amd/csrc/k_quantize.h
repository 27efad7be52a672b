// fp32 -> fp16 (round to nearest even) and fp16 -> fp32 streaming kernels
// (Section 3.1: quantize / dequantize operators; Table 1: Quantize(dtype)).
#pragma once
#include "common.h"

namespace condensa {

constexpr int kQuantThreads = 64;       // wavefront-sized workgroups measured best for these sweeps (64 vs 256)

// One float4 per thread; workgroups that lie wholly inside the array use unguarded 128-bit accesses with
// the streaming hint (nothing here is read twice).
template <bool VEC, int THREADS, typename C>
__global__ __launch_bounds__(THREADS) void k_quantize(const float* x, u64 n, u16* q, float* dq) {   // dq may be x
    const u64 wg0 = static_cast<u64>(blockIdx.x) * (THREADS * 4);
    const u64 e0 = wg0 + threadIdx.x * 4;
    const bool full = VEC && wg0 + THREADS * 4 <= n;                     // uniform
    float v[4];
    if (full) {
        const float4 t = ld4_stream(x + e0);
        v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
    } else {
        if (e0 >= n) return;
        load4<VEC>(x, e0, n, v);
    }
    u16 h[4];
    float d[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        h[k] = C::enc(v[k]);
        d[k] = C::dec(h[k]);
    }
    if (full) {
        if (q) {
            st_code4_stream(q + e0, h[0], h[1], h[2], h[3]);
        }
        if (dq) st4_stream(dq + e0, d[0], d[1], d[2], d[3]);
    } else {
        if (q) store4_u16<VEC>(q, e0, n, h);
        if (dq) store4<VEC>(dq, e0, n, d);
    }
}

// Codes only: eight elements per thread -- two loads in flight per lane and a full 128-bit store of the
// codes (measured 76% of peak against 58% with four per thread; the reverse layout, two strided 128-bit
// stores per lane, halves the rate, so the other kernels keep one float4 per thread).  Requires 16-byte
// aligned x and q.
template <int THREADS, typename C>
__global__ __launch_bounds__(THREADS) void k_quantize_codes(const float* __restrict__ x, u64 n, u16* __restrict__ q) {
    const u64 wg0 = static_cast<u64>(blockIdx.x) * (THREADS * 8);
    const u64 e0 = wg0 + threadIdx.x * 8;
    if (wg0 + THREADS * 8 <= n) {                                        // uniform
        const float4 a = ld4_stream(x + e0);
        const float4 b = ld4_stream(x + e0 + 4);
        u16x8 h;
        h[0] = C::enc(a.x); h[1] = C::enc(a.y); h[2] = C::enc(a.z); h[3] = C::enc(a.w);
        h[4] = C::enc(b.x); h[5] = C::enc(b.y); h[6] = C::enc(b.z); h[7] = C::enc(b.w);
        __builtin_nontemporal_store(h, reinterpret_cast<u16x8*>(q + e0));
    } else {
        for (int k = 0; k < 8; ++k)
            if (e0 + k < n) q[e0 + k] = C::enc(x[e0 + k]);
    }
}

template <bool VEC, int THREADS, typename C>
__global__ __launch_bounds__(THREADS) void k_dequantize(const u16* __restrict__ q, u64 n, float* __restrict__ dq) {
    const u64 wg0 = static_cast<u64>(blockIdx.x) * (THREADS * 4);
    const u64 e0 = wg0 + threadIdx.x * 4;
    const bool full = VEC && wg0 + THREADS * 4 <= n;                     // uniform
    u16 h[4];
    if (full) {
        const ushort4 t = *reinterpret_cast<const ushort4*>(q + e0);
        h[0] = t.x; h[1] = t.y; h[2] = t.z; h[3] = t.w;
    } else {
        if (e0 >= n) return;
#pragma unroll
        for (int k = 0; k < 4; ++k) h[k] = (e0 + k < n) ? q[e0 + k] : static_cast<u16>(0);
    }
    float d[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) d[k] = C::dec(h[k]);
    if (full) st4_stream(dq + e0, d[0], d[1], d[2], d[3]);
    else      store4<VEC>(dq, e0, n, d);
}

// Wide form: a wavefront takes 512 codes.  Every lane loads eight codes with one 128-bit access, the
// lanes then trade halves so that lane L holds codes 4L..4L+3 and 256+4L..256+4L+3, and writes them with
// two 128-bit stores that are contiguous across the wavefront (storing each lane's own eight values
// instead, 32 bytes apart per lane, runs at half the rate).  Requires 16-byte aligned q and dq.
template <int THREADS, typename C>
__global__ __launch_bounds__(THREADS) void k_dequantize_wide(const u16* __restrict__ q, u64 n, float* __restrict__ dq) {
    constexpr int kPerWave = 512;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const u64 wave0 = (static_cast<u64>(blockIdx.x) * (THREADS / 64) + wave) * kPerWave;
    if (wave0 >= n) return;
    if (wave0 + kPerWave <= n) {                                         // uniform over the wavefront
        typedef u32 u32x4 __attribute__((ext_vector_type(4)));
        const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(q + wave0 + lane * 8));
        // lane L needs the codes 4L..4L+3: dwords (L & 1) * 2, +1 of lane L / 2; and the same of lane 32 + L / 2
        const int src = lane >> 1;
        const bool odd = lane & 1;
        const u32 lo0 = __shfl(v[0], src, 64), lo1 = __shfl(v[1], src, 64), lo2 = __shfl(v[2], src, 64), lo3 = __shfl(v[3], src, 64);
        const u32 hi0 = __shfl(v[0], src + 32, 64), hi1 = __shfl(v[1], src + 32, 64), hi2 = __shfl(v[2], src + 32, 64), hi3 = __shfl(v[3], src + 32, 64);
        const u32 c0 = odd ? lo2 : lo0, c1 = odd ? lo3 : lo1, d0 = odd ? hi2 : hi0, d1 = odd ? hi3 : hi1;
        st4_stream(dq + wave0 + lane * 4, C::dec(static_cast<u16>(c0)), C::dec(static_cast<u16>(c0 >> 16)),
                   C::dec(static_cast<u16>(c1)), C::dec(static_cast<u16>(c1 >> 16)));
        st4_stream(dq + wave0 + 256 + lane * 4, C::dec(static_cast<u16>(d0)), C::dec(static_cast<u16>(d0 >> 16)),
                   C::dec(static_cast<u16>(d1)), C::dec(static_cast<u16>(d1 >> 16)));
    } else {
        for (int k = 0; k < 8; ++k) {
            const u64 e = wave0 + static_cast<u64>(k) * 64 + lane;
            if (e < n) dq[e] = C::dec(q[e]);
        }
    }
}

}  // namespace condensa
