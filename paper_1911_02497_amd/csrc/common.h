// Shared definitions of the gfx950 compression-step kernels: device tables, key helpers,
// chunk addressing and radix-level geometry.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/condensa.h"

typedef uint8_t u8;
typedef uint16_t u16;
typedef uint32_t u32;
typedef uint64_t u64;

namespace condensa {

constexpr int kBlock = 256;            // threads per workgroup (4 wavefronts of 64)
constexpr int kChunk = 8192;           // elements of one tensor handled as a unit of work
constexpr int kQuadsPerThread = kChunk / (kBlock * 4);   // 8 float4 per thread and chunk
constexpr int kMaxJ = CONDENSA_MAX_DENSITIES;
constexpr int kBins = 2048;            // bins of one radix level (digits are at most 11 bits)
// Elements per call.  The densest launches give one thread four elements (of tensors padded to whole
// chunks, at most 65536 of them), and a launch must stay below 2^32 threads: the runtime rejects a
// multiple of 2^32 and silently wraps anything else above it.  3 * 2^32 elements is also about what fits
// the device: an L-C step moves 20 bytes per weight.
constexpr u64 kMaxElems = static_cast<u64>(3) << 32;
constexpr int kSlotBatch = 14;         // rankings that share one sweep's LDS histograms (14 x 1024 bins x 4 B + digit table < 64 KB)

// Division of a 32-bit unsigned x by a divisor fixed on the host, by multiplication with a rounded-up
// reciprocal (Granlund & Montgomery 1994, unsigned case): with l = ceil(log2 d) and
// m = floor(2^32 (2^l - d) / d) + 1,  t = hi32(m x)  gives  x / d = (t + ((x - t) >> min(l, 1))) >> max(l - 1, 0).
struct FastDiv {
    u32 mul;
    u32 sh;                // first shift | second shift << 8
};

__host__ __device__ inline FastDiv make_fastdiv(u32 d) {   // d >= 1
    int l = 0;
    while (l < 32 && (static_cast<u64>(1) << l) < d) ++l;
    FastDiv f;
    f.mul = static_cast<u32>(((static_cast<u64>(1) << 32) * ((static_cast<u64>(1) << l) - d)) / d + 1);
    f.sh = static_cast<u32>(l < 1 ? l : 1) | (static_cast<u32>(l > 1 ? l - 1 : 0) << 8);
    return f;
}

__host__ __device__ inline u32 fast_div(u32 x, FastDiv f) {
#if defined(__HIP_DEVICE_COMPILE__)
    const u32 t = __umulhi(x, f.mul);
#else
    const u32 t = static_cast<u32>((static_cast<u64>(x) * f.mul) >> 32);
#endif
    return (t + ((x - t) >> (f.sh & 0xFFu))) >> (f.sh >> 8);
}

// One weight tensor as the kernels see it (device table, one entry per tensor plus a sentinel).
struct TensorDesc {
    const float* w;
    const float* lam;      // L-C multipliers (NULL for plain pruning)
    float* lam_out;
    float* grad;
    u64 n;                 // elements
    u64 flat_start;        // flat index of element 0
    u64 chunk_start;       // id of this tensor's first chunk
    u64 struct_start;      // id of this tensor's first structure (structure pruning)
    u32 d[4];              // structure pruning: the tensor as 4-D (leading dims 1 for lower ranks)
    u32 b[4];              // block shape; a filter / neuron is the block [1,1,1,len] of [F,1,1,len]
    u64 n_struct;          // structures in this tensor: product of ceil(d/b)
    u64 pad;               // id of this tensor's first structure chunk
    u64 reserved[2];
    FastDiv fd[7];         // reciprocals of d[1], d[2], d[3], b[0], b[1], b[2], b[3] (structure pruning)
    u64 reserved2;
};
static_assert(sizeof(TensorDesc) == 192, "TensorDesc layout");
enum { kDivD1 = 0, kDivD2, kDivD3, kDivB0, kDivB1, kDivB2, kDivB3 };

struct OutDesc {           // outputs of tensor t for density j, entry j * n_tensors + t
    float* theta;
    u16* theta16;
    u8* mask;
    u64 pad;
};

// State of a ranking as the radix-level kernels hand it on: the level kernels of a GLOBAL-scope ranking do
// not wait for a separate bin-search launch -- every workgroup of the kernel for level L folds the finished
// histogram of level L - 1 into the state itself (all workgroups get the same result), and workgroup 0 stores
// it for the kernel of level L + 1.  The stores alternate between two places so that no workgroup can read a
// state while another one of the same kernel replaces it.
struct SlotStep {
    u64 prefix;            // key bits decided so far
    u64 remaining;         // 1-based descending rank still to resolve inside the prefix
    u64 n_tie;             // keys in the bin chosen last
    u32 state;
    u32 need_tie;
};

// State of one ranking (one density of one group).  Filled by the host, advanced level by level.  The fields
// before `step` are only ever written by the host or by kernels that run one workgroup per ranking.
struct Slot {
    u64 prefix;            // key bits decided so far
    u64 remaining;         // 1-based descending rank still to resolve inside the prefix
    u64 k;
    u64 n;
    u64 n_tie;
    u64 tie_end;
    u64 lo, hi;            // sampled key window (window path)
    u32 state;             // kInactive (k == 0), kSelecting, kDone
    u32 need_tie;          // index search among ties required
    u32 path;
    u32 level_begin;       // radix levels below this one are already decided by the prefix
    u32 rank_rule;         // 0: `remaining` is given.  Else this ranking bounds the threshold of another one on a
                           // sample whose size is only known on the device: kRankHi / kRankLo / kRankMid
    u32 margin16;          // rank_rule != 0: half-width of the window in 1/16 standard deviations of the sample rank
    double p;              // rank_rule != 0: k / n of the ranking that is bounded
    SlotStep step[2];      // step[L & 1]: state on entering level L, stored by the kernel of level L (L > level_begin)
};
static_assert(sizeof(SlotStep) == 32 && sizeof(Slot) == 160, "Slot layout");
enum : u32 { kRankGiven = 0, kRankHi = 1, kRankLo = 2, kRankMid = 3 };

enum : u32 { kInactive = 0, kSelecting = 1, kDone = 2, kFailed = 3 };

// Radix level geometry for keys of `key_bits` significant bits (31 for |fp32|, 63 for fp64 sums,
// fewer for index keys): ceil(key_bits / 11) levels of at most 11 bits, most significant first.
struct Level {
    int shift;             // position of the digit
    int bits;              // digit width
    int hi_shift;          // shift + bits: key >> hi_shift must equal prefix >> hi_shift
};

__host__ __device__ inline int n_levels(int key_bits) { return (key_bits + 10) / 11; }

// Digits are as even as possible, wider ones first: 31 -> 11,10,10; 63 -> 11,11,11,10,10,10.
__host__ __device__ inline Level level_of(int key_bits, int level) {
    const int nl = n_levels(key_bits);
    const int base = key_bits / nl, extra = key_bits % nl;
    Level L;
    L.bits = base + (level < extra ? 1 : 0);
    L.hi_shift = key_bits - (level * base + (level < extra ? level : extra));
    L.shift = L.hi_shift - L.bits;
    return L;
}

__device__ inline u32 mag_key(float x) { return __float_as_uint(x) & 0x7FFFFFFFu; }

// v = w - lambda / mu in binary32, one rounding per operation (no contraction).
__device__ inline float lc_shift(float w, float lam, float mu) {
    const float t = __fdiv_rn(lam, mu);
    return __fsub_rn(w, t);
}

// 128-bit accesses with the streaming (non-temporal) hint, for data that this call touches for the last
// time: results that nothing re-reads before they leave the caches anyway, inputs on their final pass.
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned short u16x8 __attribute__((ext_vector_type(8)));
__device__ inline float4 ld4_stream(const float* p) {
    const f32x4 t = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p));
    return make_float4(t.x, t.y, t.z, t.w);
}
// The stores carry the system-scope bits together with the non-temporal one (write straight through, keep
// nothing): on the L-C mix of 2 streams read and 3 written this measured 1.5-2 % faster than the non-temporal
// bit alone, which is all that __builtin_nontemporal_store sets.  They are raw buffer stores, the one store
// form whose cache-policy bits the compiler exposes (sc0 = 1, nt = 2, sc1 = 16), so the compiler schedules them
// and keeps the wait states that the hardware wants between a wide store and a rewrite of its data registers
// -- nothing here is hand-written assembly.  The buffer descriptor is built around the address of the
// wavefront's first active lane and every lane adds its distance from it; all callers store to addresses that
// ascend with the lane, within a few KB.  A lane that broke that rule would fall outside the descriptor's
// 2 GB range and its store would be dropped, which the parity tests would show.
// Building the library with -DCONDENSA_PLAIN_STREAM_STORES swaps in the compiler's own non-temporal global
// stores, to cross-check a parity failure against.
constexpr int kStreamPolicy = 1 | 2 | 16;
__device__ inline u32 stream_offset(const void* p, __amdgpu_buffer_rsrc_t* rsrc) {
    const u64 a = reinterpret_cast<u64>(p);
    // (the builtin returns a signed int: without the casts its lower half would be sign-extended into the upper one)
    const u32 base_hi = static_cast<u32>(__builtin_amdgcn_readfirstlane(static_cast<int>(a >> 32)));
    const u32 base_lo = static_cast<u32>(__builtin_amdgcn_readfirstlane(static_cast<int>(a)));
    const u64 base = (static_cast<u64>(base_hi) << 32) | static_cast<u64>(base_lo);
    *rsrc = __builtin_amdgcn_make_buffer_rsrc(reinterpret_cast<void*>(base), 0, 0x7FFFFFFF, 0x00020000);
    return static_cast<u32>(a - base);
}
typedef u32 u32x2 __attribute__((ext_vector_type(2)));
typedef u32 u32x4 __attribute__((ext_vector_type(4)));
__device__ inline void st_words4_stream(void* p, u32x4 t) {          // sixteen bytes (p 16-byte aligned)
#if defined(CONDENSA_PLAIN_STREAM_STORES)
    __builtin_nontemporal_store(t, reinterpret_cast<u32x4*>(p));
#else
    __amdgpu_buffer_rsrc_t r;
    const u32 off = stream_offset(p, &r);
    __builtin_amdgcn_raw_buffer_store_b128(t, r, off, 0, kStreamPolicy);
#endif
}
__device__ inline void st4_stream(float* p, float a, float b, float c, float d) {
    u32x4 t;
    t.x = __float_as_uint(a); t.y = __float_as_uint(b); t.z = __float_as_uint(c); t.w = __float_as_uint(d);
    st_words4_stream(p, t);
}
// Four mask bytes / four 16-bit codes as one store (p 4- / 8-byte aligned).
__device__ inline void st_mask4_stream(u8* p, u8 a, u8 b, u8 c, u8 d) {
    const u32 t = static_cast<u32>(a) | (static_cast<u32>(b) << 8) | (static_cast<u32>(c) << 16) | (static_cast<u32>(d) << 24);
#if defined(CONDENSA_PLAIN_STREAM_STORES)
    __builtin_nontemporal_store(t, reinterpret_cast<u32*>(p));
#else
    __amdgpu_buffer_rsrc_t r;
    const u32 off = stream_offset(p, &r);
    __builtin_amdgcn_raw_buffer_store_b32(t, r, off, 0, kStreamPolicy);
#endif
}
__device__ inline void st_code4_stream(u16* p, u16 a, u16 b, u16 c, u16 d) {
    u32x2 t;
    t.x = static_cast<u32>(a) | (static_cast<u32>(b) << 16);
    t.y = static_cast<u32>(c) | (static_cast<u32>(d) << 16);
#if defined(CONDENSA_PLAIN_STREAM_STORES)
    __builtin_nontemporal_store(t, reinterpret_cast<u32x2*>(p));
#else
    __amdgpu_buffer_rsrc_t r;
    const u32 off = stream_offset(p, &r);
    __builtin_amdgcn_raw_buffer_store_b64(t, r, off, 0, kStreamPolicy);
#endif
}

// Loads up to four consecutive elements e0 .. e0+3 of an n-element array; missing ones read 0.
template <bool VEC>
__device__ inline void load4(const float* __restrict__ p, u64 e0, u64 n, float v[4]) {
    if (VEC && e0 + 4 <= n) {
        const float4 t = *reinterpret_cast<const float4*>(p + e0);
        v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
    } else {
#pragma unroll
        for (int k = 0; k < 4; ++k) v[k] = (e0 + k < n) ? p[e0 + k] : 0.0f;
    }
}

template <bool VEC>
__device__ inline void store4(float* __restrict__ p, u64 e0, u64 n, const float v[4]) {
    if (VEC && e0 + 4 <= n) {
        *reinterpret_cast<float4*>(p + e0) = make_float4(v[0], v[1], v[2], v[3]);
    } else {
#pragma unroll
        for (int k = 0; k < 4; ++k) if (e0 + k < n) p[e0 + k] = v[k];
    }
}

template <bool VEC>
__device__ inline void store4_u8(u8* __restrict__ p, u64 e0, u64 n, const u8 v[4]) {
    if (VEC && e0 + 4 <= n) {
        *reinterpret_cast<uchar4*>(p + e0) = make_uchar4(v[0], v[1], v[2], v[3]);
    } else {
#pragma unroll
        for (int k = 0; k < 4; ++k) if (e0 + k < n) p[e0 + k] = v[k];
    }
}

template <bool VEC>
__device__ inline void store4_u16(u16* __restrict__ p, u64 e0, u64 n, const u16 v[4]) {
    if (VEC && e0 + 4 <= n) {
        *reinterpret_cast<ushort4*>(p + e0) = make_ushort4(v[0], v[1], v[2], v[3]);
    } else {
#pragma unroll
        for (int k = 0; k < 4; ++k) if (e0 + k < n) p[e0 + k] = v[k];
    }
}

// Tensor that owns chunk c: largest t with chunk_start[t] <= c (table has a sentinel at n_tensors).
__device__ inline int tensor_of_chunk(const TensorDesc* __restrict__ td, int n_tensors, u64 c) {
    int lo = 0, hi = n_tensors - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (td[mid].chunk_start <= c) lo = mid; else hi = mid - 1;
    }
    return lo;
}

// binary32 -> binary16 bits, round to nearest even (overflow to inf, gradual underflow, quiet NaN
// with the sign and top ten payload bits).  Numbers take the conversion instruction (round to nearest even and
// binary16 subnormals are the modes every kernel here is compiled and launched with; the parity tests sweep
// every exponent band, ties and subnormals included, against the oracle's integer arithmetic): inside the L-C
// sweep the integer form below cost more instructions than the memory traffic could hide.  NaNs keep the
// integer form, which fixes their payload.  -DCONDENSA_INTEGER_F16 builds the integer form throughout.
__device__ inline u16 f32_to_f16_rne(float x) {
    const u32 b = __float_as_uint(x);
    const u32 sign = (b >> 16) & 0x8000u;
    const u32 a = b & 0x7FFFFFFFu;
#if !defined(CONDENSA_INTEGER_F16)
    if (a <= 0x7F800000u) {
        const _Float16 hw = static_cast<_Float16>(x);
        u16 bits;
        __builtin_memcpy(&bits, &hw, sizeof(bits));
        return bits;
    }
#endif
    u32 h;
    if (a >= 0x47800000u) {                                  // |x| >= 2^16, inf or NaN
        h = (a > 0x7F800000u) ? (0x7E00u | ((a >> 13) & 0x3FFu)) : 0x7C00u;
    } else if (a >= 0x38800000u) {                           // normal binary16 range
        const u32 r = a - 0x38000000u;                       // rebias exponent by 112
        h = r >> 13;
        const u32 rem = r & 0x1FFFu;
        h += (rem > 0x1000u) | ((rem == 0x1000u) & (h & 1u));
    } else if (a >= 0x33000000u) {                           // subnormal binary16 (2^-25 <= |x| < 2^-14)
        const u32 e = a >> 23;                               // 102 .. 112
        const u32 m = (a & 0x007FFFFFu) | 0x00800000u;
        const u32 s = 126u - e;                              // 14 .. 24
        h = m >> s;
        const u32 rem = m & ((1u << s) - 1u);
        const u32 half = 1u << (s - 1u);
        h += (rem > half) | ((rem == half) & (h & 1u));
    } else {
        h = 0u;
    }
    return static_cast<u16>(sign | h);
}

// exact widening binary16 -> binary32 (numbers by the conversion instruction, infinities and NaN patterns bit by bit)
__device__ inline float f16_bits_to_f32(u16 hb) {
    const u32 h = hb;
    const u32 sign = (h & 0x8000u) << 16;
    const u32 e = (h >> 10) & 0x1Fu;
    const u32 m = h & 0x3FFu;
#if !defined(CONDENSA_INTEGER_F16)
    if (e != 31u) {
        _Float16 hw;
        __builtin_memcpy(&hw, &hb, sizeof(hw));
        return static_cast<float>(hw);
    }
#endif
    u32 out;
    if (e == 31u) {
        out = sign | 0x7F800000u | (m << 13);
    } else if (e != 0u) {
        out = sign | ((e + 112u) << 23) | (m << 13);
    } else if (m == 0u) {
        out = sign;
    } else {
        const int lz = __clz(static_cast<int>(m)) - 21;      // shifts needed to reach bit 10
        const u32 mm = (m << lz) & 0x3FFu;
        out = sign | (static_cast<u32>(113 - lz) << 23) | (mm << 13);
    }
    return __uint_as_float(out);
}

// bfloat16 (upper half of binary32), round to nearest even: add half of the dropped range, less one when the
// kept part is even (so that an exact tie does not carry); a carry runs into the exponent and the largest
// finite values become infinity.  NaN keeps sign and upper payload, quiet bit set.
__device__ inline u16 f32_to_bf16_rne(float x) {
    const u32 u = __float_as_uint(x);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return static_cast<u16>((u >> 16) | 0x0040u);
    return static_cast<u16>((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
}

__device__ inline float bf16_bits_to_f32(u16 hb) { return __uint_as_float(static_cast<u32>(hb) << 16); }

// The 16-bit codecs of the quantize kernels.
struct CodecF16 {
    static __device__ inline u16 enc(float x) { return f32_to_f16_rne(x); }
    static __device__ inline float dec(u16 h) { return f16_bits_to_f32(h); }
};
struct CodecBF16 {
    static __device__ inline u16 enc(float x) { return f32_to_bf16_rne(x); }
    static __device__ inline float dec(u16 h) { return bf16_bits_to_f32(h); }
};

// 8-bit floating point with EXP exponent bits, MAN fraction bits and the given bias (OCP 8-bit floating
// point formats: E4M3 has no infinity and one NaN pattern per sign, E5M2 is IEEE-like).  Round to nearest
// even in integer arithmetic on the binary32 pattern (normal results) or by an exact power-of-two scaling
// and the hardware's round-to-nearest-even integer conversion (subnormal results); finite values beyond the
// largest finite code saturate to it; E5M2 keeps infinities, E4M3 saturates them; NaN keeps its sign.
template <int EXP, int MAN, int BIAS, bool HAS_INF>
struct CodecFP8 {
    static constexpr u32 kMaxCode = HAS_INF ? ((((1u << EXP) - 1u) << MAN) - 1u) : 0x7Eu;
    static constexpr u32 kInfCode = ((1u << EXP) - 1u) << MAN;
    static constexpr int kEmin = 1 - BIAS;                            // exponent of the smallest normal value
    static __device__ inline u8 enc(float x) {
        const u32 u = __float_as_uint(x);
        const u32 sign = (u >> 24) & 0x80u;
        const u32 a = u & 0x7FFFFFFFu;
        if (a > 0x7F800000u) return static_cast<u8>(sign | (HAS_INF ? (kInfCode | (1u << (MAN - 1))) : 0x7Fu));
        if (a == 0x7F800000u) return static_cast<u8>(sign | (HAS_INF ? kInfCode : kMaxCode));
        const int e = static_cast<int>(a >> 23) - 127;
        u32 code;
        if (e >= kEmin) {
            constexpr int SH = 23 - MAN;
            const u32 r = a + ((1u << (SH - 1)) - 1u) + ((a >> SH) & 1u);      // ties to even; a carry runs into the exponent
            code = (r >> SH) - (static_cast<u32>(127 - BIAS) << MAN);
        } else {
            // below the smallest normal value the codes are multiples of 2^(kEmin - MAN): 0 .. 2^MAN
            code = static_cast<u32>(__float2int_rn(__uint_as_float(a) * __uint_as_float(static_cast<u32>(127 + MAN - kEmin) << 23)));
        }
        if (code > kMaxCode) code = kMaxCode;
        return static_cast<u8>(sign | code);
    }
    static __device__ inline float dec(u8 c) {
        const u32 sign = static_cast<u32>(c & 0x80u) << 24;
        const u32 mag = c & 0x7Fu;
        const u32 ex = mag >> MAN, m = mag & ((1u << MAN) - 1u);
        if (mag > kMaxCode) return __uint_as_float(sign | ((HAS_INF && mag == kInfCode) ? 0x7F800000u : 0x7FC00000u));
        if (ex == 0) {
            const float v = static_cast<float>(m) * __uint_as_float(static_cast<u32>(127 + kEmin - MAN) << 23);   // exact
            return __uint_as_float(sign | __float_as_uint(v));
        }
        return __uint_as_float(sign | ((ex + static_cast<u32>(127 - BIAS)) << 23) | (m << (23 - MAN)));
    }
};
typedef CodecFP8<4, 3, 7, false> CodecE4M3;
typedef CodecFP8<5, 2, 15, true> CodecE5M2;

}  // namespace condensa
