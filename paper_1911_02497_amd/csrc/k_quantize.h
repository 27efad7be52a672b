// fp32 -> 16-bit / 8-bit floating point (round to nearest even) and back: streaming kernels
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

// Codes only: a wavefront takes 512 elements.  Every lane issues two 128-bit loads that are contiguous
// across the wavefront and packs two 64-bit words of codes; the lanes then trade words so that lane L
// holds the codes of elements 8 L .. 8 L + 7 and stores them with one 128-bit access (77 % of peak; with
// each lane loading its own eight elements, 32 bytes apart per lane, 76 %; with four elements per thread
// and 8-byte stores 58 %; two strided 128-bit stores per lane halve the rate, so the kernels that also
// write the widened values keep one float4 per thread).  Requires 16-byte aligned x and q.
template <int THREADS, typename C>
__global__ __launch_bounds__(THREADS) void k_quantize_codes(const float* __restrict__ x, u64 n, u16* __restrict__ q) {
    constexpr int kPerWave = 512;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const u64 wave0 = (static_cast<u64>(blockIdx.x) * (THREADS / 64) + wave) * kPerWave;
    if (wave0 >= n) return;
    if (wave0 + kPerWave <= n) {                                         // uniform over the wavefront
        u32 lo[2], hi[2];
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            const float4 v = ld4_stream(x + wave0 + k * 256 + lane * 4);
            lo[k] = static_cast<u32>(C::enc(v.x)) | (static_cast<u32>(C::enc(v.y)) << 16);
            hi[k] = static_cast<u32>(C::enc(v.z)) | (static_cast<u32>(C::enc(v.w)) << 16);
        }
        // 64-bit word j of the wavefront (elements 4 j .. 4 j + 3) sits in (lo, hi)[j / 64] of lane j % 64;
        // lane L wants words 2 L and 2 L + 1
        const int kk = lane >> 5, src = (lane * 2) & 63;
        u32x4 out;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const u32 a0 = __shfl(lo[0], src + i, 64), a1 = __shfl(lo[1], src + i, 64);
            const u32 b0 = __shfl(hi[0], src + i, 64), b1 = __shfl(hi[1], src + i, 64);
            out[2 * i] = kk == 0 ? a0 : a1;
            out[2 * i + 1] = kk == 0 ? b0 : b1;
        }
        st_words4_stream(q + wave0 + lane * 8, out);
    } else {
        for (int k = 0; k < 8; ++k) {
            const u64 e = wave0 + static_cast<u64>(k) * 64 + lane;
            if (e < n) q[e] = C::enc(x[e]);
        }
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

// ---- 8-bit codes ---------------------------------------------------------------------------------------
// One float4 per thread, four codes stored as one 32-bit word.
template <bool VEC, int THREADS, typename C>
__global__ __launch_bounds__(THREADS) void k_quantize8(const float* x, u64 n, u8* q, float* dq) {   // dq may be x
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
    u8 h[4];
    float d[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        h[k] = C::enc(v[k]);
        d[k] = C::dec(h[k]);
    }
    if (full) {
        if (q) st_mask4_stream(q + e0, h[0], h[1], h[2], h[3]);
        if (dq) st4_stream(dq + e0, d[0], d[1], d[2], d[3]);
    } else {
        if (q) store4_u8<VEC>(q, e0, n, h);
        if (dq) store4<VEC>(dq, e0, n, d);
    }
}

// Codes only: a wavefront takes 1024 elements.  Every lane issues four 128-bit loads that are contiguous
// across the wavefront and packs four 32-bit words of codes; the lanes then trade words so that lane L
// holds the codes of elements 16 L .. 16 L + 15 and stores them with one 128-bit access (loading each
// lane's own sixteen elements instead leaves every cache line to four separate load instructions).
// Requires 16-byte aligned x and q.
template <int THREADS, typename C>
__global__ __launch_bounds__(THREADS) void k_quantize8_codes(const float* __restrict__ x, u64 n, u8* __restrict__ q) {
    constexpr int kPerWave = 1024;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const u64 wave0 = (static_cast<u64>(blockIdx.x) * (THREADS / 64) + wave) * kPerWave;
    if (wave0 >= n) return;
    if (wave0 + kPerWave <= n) {                                         // uniform over the wavefront
        u32 w[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const float4 v = ld4_stream(x + wave0 + k * 256 + lane * 4);
            w[k] = static_cast<u32>(C::enc(v.x)) | (static_cast<u32>(C::enc(v.y)) << 8) |
                   (static_cast<u32>(C::enc(v.z)) << 16) | (static_cast<u32>(C::enc(v.w)) << 24);
        }
        // word j of the wavefront (elements 4 j .. 4 j + 3) sits in w[j / 64] of lane j % 64; lane L wants words 4 L .. 4 L + 3
        const int kk = lane >> 4, src = (lane * 4) & 63;
        u32x4 out;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const u32 t0 = __shfl(w[0], src + i, 64), t1 = __shfl(w[1], src + i, 64);
            const u32 t2 = __shfl(w[2], src + i, 64), t3 = __shfl(w[3], src + i, 64);
            out[i] = kk == 0 ? t0 : (kk == 1 ? t1 : (kk == 2 ? t2 : t3));
        }
        st_words4_stream(q + wave0 + lane * 16, out);
    } else {
        for (int k = 0; k < 16; ++k) {
            const u64 e = wave0 + static_cast<u64>(k) * 64 + lane;
            if (e < n) q[e] = C::enc(x[e]);
        }
    }
}

// Four codes (one 32-bit load) per thread, one 128-bit store.
template <bool VEC, int THREADS, typename C>
__global__ __launch_bounds__(THREADS) void k_dequantize8(const u8* __restrict__ q, u64 n, float* __restrict__ dq) {
    const u64 wg0 = static_cast<u64>(blockIdx.x) * (THREADS * 4);
    const u64 e0 = wg0 + threadIdx.x * 4;
    const bool full = VEC && wg0 + THREADS * 4 <= n;                     // uniform
    u8 h[4];
    if (full) {
        const u32 t = __builtin_nontemporal_load(reinterpret_cast<const u32*>(q + e0));
        h[0] = static_cast<u8>(t); h[1] = static_cast<u8>(t >> 8); h[2] = static_cast<u8>(t >> 16); h[3] = static_cast<u8>(t >> 24);
    } else {
        if (e0 >= n) return;
#pragma unroll
        for (int k = 0; k < 4; ++k) h[k] = (e0 + k < n) ? q[e0 + k] : static_cast<u8>(0);
    }
    float d[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) d[k] = C::dec(h[k]);
    if (full) st4_stream(dq + e0, d[0], d[1], d[2], d[3]);
    else      store4<VEC>(dq, e0, n, d);
}

// Wide form: a wavefront takes 1024 codes.  Every lane loads sixteen codes with one 128-bit access, the
// lanes trade words so that lane L holds the codes of elements 256 s + 4 L .. + 3 for s = 0..3, and
// writes them with four 128-bit stores that are contiguous across the wavefront.  Requires 16-byte
// aligned q and dq.
template <int THREADS, typename C>
__global__ __launch_bounds__(THREADS) void k_dequantize8_wide(const u8* __restrict__ q, u64 n, float* __restrict__ dq) {
    constexpr int kPerWave = 1024;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const u64 wave0 = (static_cast<u64>(blockIdx.x) * (THREADS / 64) + wave) * kPerWave;
    if (wave0 >= n) return;
    if (wave0 + kPerWave <= n) {                                         // uniform over the wavefront
        const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(q + wave0 + lane * 16));
        const int d = lane & 3;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const int src = s * 16 + (lane >> 2);                        // its word d covers elements 256 s + 4 L ..
            const u32 t0 = __shfl(v[0], src, 64), t1 = __shfl(v[1], src, 64), t2 = __shfl(v[2], src, 64), t3 = __shfl(v[3], src, 64);
            const u32 word = d == 0 ? t0 : (d == 1 ? t1 : (d == 2 ? t2 : t3));
            st4_stream(dq + wave0 + s * 256 + lane * 4, C::dec(static_cast<u8>(word)), C::dec(static_cast<u8>(word >> 8)),
                       C::dec(static_cast<u8>(word >> 16)), C::dec(static_cast<u8>(word >> 24)));
        }
    } else {
        for (int k = 0; k < 16; ++k) {
            const u64 e = wave0 + static_cast<u64>(k) * 64 + lane;
            if (e < n) dq[e] = C::dec(q[e]);
        }
    }
}

}  // namespace condensa
