// fp32 -> fp16 (round to nearest even) and fp16 -> fp32 streaming kernels
// (Section 3.1: quantize / dequantize operators; Table 1: Quantize(dtype)).
#pragma once
#include "common.h"

namespace condensa {

template <bool VEC>
__global__ __launch_bounds__(kBlock) void k_quantize(const float* x, u64 n, u16* q, float* dq) {
    const u64 n_quads = (n + 3) / 4;
    const u64 stride = static_cast<u64>(gridDim.x) * kBlock;
    for (u64 i = static_cast<u64>(blockIdx.x) * kBlock + threadIdx.x; i < n_quads; i += stride) {
        const u64 e0 = i * 4;
        float v[4];
        load4<VEC>(x, e0, n, v);
        u16 h[4];
        float d[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            h[k] = f32_to_f16_rne(v[k]);
            d[k] = f16_bits_to_f32(h[k]);
        }
        if (q) store4_u16<VEC>(q, e0, n, h);
        if (dq) store4<VEC>(dq, e0, n, d);
    }
}

template <bool VEC>
__global__ __launch_bounds__(kBlock) void k_dequantize(const u16* q, u64 n, float* dq) {
    const u64 n_quads = (n + 3) / 4;
    const u64 stride = static_cast<u64>(gridDim.x) * kBlock;
    for (u64 i = static_cast<u64>(blockIdx.x) * kBlock + threadIdx.x; i < n_quads; i += stride) {
        const u64 e0 = i * 4;
        u16 h[4];
        if (VEC && e0 + 4 <= n) {
            const ushort4 t = *reinterpret_cast<const ushort4*>(q + e0);
            h[0] = t.x; h[1] = t.y; h[2] = t.z; h[3] = t.w;
        } else {
#pragma unroll
            for (int k = 0; k < 4; ++k) h[k] = (e0 + k < n) ? q[e0 + k] : static_cast<u16>(0);
        }
        float d[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) d[k] = f16_bits_to_f32(h[k]);
        store4<VEC>(dq, e0, n, d);
    }
}

}  // namespace condensa
