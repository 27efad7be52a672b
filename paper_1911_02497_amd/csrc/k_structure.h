// Structure pruning: per-filter / per-block sums of squares, ranking of the aggregates, structure
// masks, kept-index lists and the element-wise apply.
// Table 1: FilterPrune (filters, seen as 3-D blocks, are aggregated and pruned), BlockPrune (blocks of any
// dimensionality and a given size); Section 3.1: the schemes aggregate filters, neurons and blocks.
#pragma once
#include "k_apply.h"
#include "k_select.h"

namespace condensa {

struct StructArgs {
    const TensorDesc* td;
    Slot* slots;
    u64* histx;            // [n_slots][kBins]
    u32* tiecnt;           // [n_schunks]
    Control* ctl;
    u64* keys;             // [F] sign-less binary64 patterns of the aggregates
    u8* smask;             // [F]
    u32* sblock;           // kept structures per tile of kMaskTile structures, then its exclusive scan
    const u32* chunk_map;  // [n_chunks] tensor that owns each element chunk
    u64 F;
    u64 n_schunks;
    u64 n_chunks;
    int n_tensors;
    int per_tensor;
    // GLOBAL scope, groups too large for k_struct_small: one histogram per radix level (histx[level]), and each
    // level's kernel folds in the level before it (wave_enter_level) instead of a k_scan_level launch in between
    int merged;
    u64* hist_base;        // merged form: first histogram of the workspace, the origin of the coarse sums
    u64* coarse;           // merged form: kCoarse sums per histogram
    int only_failed;       // 1: the levels over all aggregates are the fallback of the one-sweep form's short
                           // ranking (k_struct_fused.h) and return at once unless that one failed
};

// merged form: histogram of radix level `level` of the one ranking, and its coarse sums
__device__ inline u64* struct_hist(const StructArgs& a, int level) { return a.histx + static_cast<u64>(level) * kBins; }
__device__ inline u64* struct_coarse(const StructArgs& a, int level) { return coarse_of(a.hist_base, a.coarse, struct_hist(a, level)); }

__device__ inline int tensor_of_struct(const TensorDesc* __restrict__ td, int n_tensors, u64 u) {
    int lo = 0, hi = n_tensors - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (td[mid].struct_start <= u) lo = mid; else hi = mid - 1;
    }
    return lo;
}

__device__ inline int tensor_of_schunk(const TensorDesc* __restrict__ td, int n_tensors, u64 c) {
    int lo = 0, hi = n_tensors - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (td[mid].pad <= c) lo = mid; else hi = mid - 1;
    }
    return lo;
}

// One thread per structure; squares are added in binary64 in memory order (row-major inside an
// n-D block, edge blocks clipped), so the aggregate does not depend on the launch shape.  x*x is
// exact in binary64.
__global__ __launch_bounds__(kBlock) void k_struct_sumsq(StructArgs a, double* sumsq, float* norms) {
    const u64 u = static_cast<u64>(blockIdx.x) * kBlock + threadIdx.x;
    if (u >= a.F) return;
    const int t = tensor_of_struct(a.td, a.n_tensors, u);
    const TensorDesc& td = a.td[t];
    const u32 d0 = td.d[0], d1 = td.d[1], d2 = td.d[2], d3 = td.d[3];
    const u32 b0 = td.b[0], b1 = td.b[1], b2 = td.b[2], b3 = td.b[3];
    const u32 G1 = (d1 + b1 - 1) / b1, G2 = (d2 + b2 - 1) / b2, G3 = (d3 + b3 - 1) / b3;
    u64 s = u - td.struct_start;
    const u32 g3 = static_cast<u32>(s % G3); s /= G3;
    const u32 g2 = static_cast<u32>(s % G2); s /= G2;
    const u32 g1 = static_cast<u32>(s % G1);
    const u32 g0 = static_cast<u32>(s / G1);
    const u32 x0e = (g0 * b0 + b0 < d0) ? g0 * b0 + b0 : d0;
    const u32 x1e = (g1 * b1 + b1 < d1) ? g1 * b1 + b1 : d1;
    const u32 x2e = (g2 * b2 + b2 < d2) ? g2 * b2 + b2 : d2;
    const u32 x3b = g3 * b3;
    const u32 len = (x3b + b3 < d3) ? b3 : d3 - x3b;
    const bool aligned = (reinterpret_cast<uintptr_t>(td.w) & 15u) == 0;
    double acc = 0.0;
    for (u32 x0 = g0 * b0; x0 < x0e; ++x0)
        for (u32 x1 = g1 * b1; x1 < x1e; ++x1)
            for (u32 x2 = g2 * b2; x2 < x2e; ++x2) {
                const u64 off = ((static_cast<u64>(x0) * d1 + x1) * d2 + x2) * d3 + x3b;
                const float* row = td.w + off;
                if (aligned && ((off | len) & 3u) == 0) {
                    for (u32 x = 0; x < len; x += 4) {
                        const float4 v = *reinterpret_cast<const float4*>(row + x);   // no streaming hint: the lanes of a
                        acc = acc + static_cast<double>(v.x) * static_cast<double>(v.x); // wavefront share cache lines here
                        acc = acc + static_cast<double>(v.y) * static_cast<double>(v.y);
                        acc = acc + static_cast<double>(v.z) * static_cast<double>(v.z);
                        acc = acc + static_cast<double>(v.w) * static_cast<double>(v.w);
                    }
                } else {
                    for (u32 x = 0; x < len; ++x) {
                        const double v = static_cast<double>(row[x]);
                        acc = acc + v * v;
                    }
                }
            }
    a.keys[u] = static_cast<u64>(__double_as_longlong(acc)) & 0x7FFFFFFFFFFFFFFFull;
    if (sumsq) sumsq[u] = acc;
    if (norms) norms[u] = static_cast<float>(sqrt(acc));
}

// Tensor that owns structure u: a proportional guess (exact when the tensors hold equal numbers of
// structures) checked against the neighbouring starts, else the binary search.
__device__ inline int tensor_of_struct_guess(const TensorDesc* __restrict__ td, int n_tensors, u64 F, u64 u) {
    int g = static_cast<int>(static_cast<float>(u) * (static_cast<float>(n_tensors) / static_cast<float>(F)));
    g = g < 0 ? 0 : (g > n_tensors - 1 ? n_tensors - 1 : g);
    const u64 lo = td[g].struct_start;
    const u64 hi = (g + 1 < n_tensors) ? td[g + 1].struct_start : F;
    if (lo <= u && u < hi) return g;
    return tensor_of_struct(td, n_tensors, u);
}

__device__ inline double add_squares(double acc, const float4& v) {
    acc = acc + static_cast<double>(v.x) * static_cast<double>(v.x);
    acc = acc + static_cast<double>(v.y) * static_cast<double>(v.y);
    acc = acc + static_cast<double>(v.z) * static_cast<double>(v.z);
    acc = acc + static_cast<double>(v.w) * static_cast<double>(v.w);
    return acc;
}

// 2-D blocks of width 4 Q (Q = 1, 2, 4, 8) that tile their matrices exactly, rows 16-byte aligned, fewer
// than 2^32 elements per tensor.  One thread per block; the loads of 16 / Q block rows are issued
// together before their squares are added in row-major order -- the same additions in the same order
// as k_struct_sumsq.  Q = 2: where the 64 blocks of a wavefront lie in one block row, lane l fetches the
// l-th and the (64 + l)-th float4 of the run (two fully used 1 KB loads per matrix row, so the streaming
// hint is safe), even lanes own the run's blocks 0..31 and odd lanes blocks 32..63, and neighbouring
// lanes trade the halves they fetched for each other.
template <int Q>
__global__ __launch_bounds__(kBlock) void k_struct_sumsq_tiles(StructArgs a, double* sumsq, float* norms) {
    constexpr int G = 16 / Q;                                // block rows per group of loads
    const u32 lane = threadIdx.x & 63u;
    const u64 wb = static_cast<u64>(blockIdx.x) * kBlock + (threadIdx.x & ~63u);   // the wavefront's first block
    if (wb >= a.F) return;
    double acc = 0.0;
    u64 u = wb + lane;
    bool run = false;
    if (Q == 2 && wb + 64 <= a.F) {                          // every lane computes the same values here
        const int t = tensor_of_struct_guess(a.td, a.n_tensors, a.F, wb);
        const TensorDesc& td = a.td[t];
        const u64 s0 = wb - td.struct_start;
        if (s0 + 64 <= td.n_struct) {
            const u32 d3 = td.d[3], b2 = td.b[2];
            const u32 G3 = fast_div(d3, td.fd[kDivB3]);
            const u32 s32 = static_cast<u32>(s0);
            const u32 g2 = s32 / G3, g3 = s32 - g2 * G3;
            if (g3 + 64 <= G3) {
                run = true;
                const u32 half = lane & 1u;
                u = wb + (lane >> 1) + (half ? 32u : 0u);
                const float* p = td.w + static_cast<u64>(g2) * b2 * d3 + static_cast<u64>(g3) * 8u + lane * 4u;
                for (u32 r0 = 0; r0 < b2; r0 += G) {
                    float4 va[G], vb[G];
#pragma unroll
                    for (int g = 0; g < G; ++g)
                        if (r0 + g < b2) {
                            const float* q = p + static_cast<u64>(r0 + g) * d3;
                            va[g] = ld4_stream(q);
                            vb[g] = ld4_stream(q + 256);
                        }
#pragma unroll
                    for (int g = 0; g < G; ++g) {
                        if (r0 + g < b2) {                   // the same for every lane: one tensor, one block height
                            const float4 send = half ? va[g] : vb[g];
                            float4 recv;
                            recv.x = __shfl_xor(send.x, 1); recv.y = __shfl_xor(send.y, 1);
                            recv.z = __shfl_xor(send.z, 1); recv.w = __shfl_xor(send.w, 1);
                            acc = add_squares(acc, half ? recv : va[g]);
                            acc = add_squares(acc, half ? vb[g] : recv);
                        }
                    }
                }
            }
        }
    }
    if (!run) {
        if (u >= a.F) return;
        const int t = tensor_of_struct_guess(a.td, a.n_tensors, a.F, u);
        const TensorDesc& td = a.td[t];
        const u32 d3 = td.d[3], b2 = td.b[2];
        const u32 G3 = fast_div(d3, td.fd[kDivB3]);
        const u32 s = static_cast<u32>(u - td.struct_start);
        const u32 g2 = s / G3, g3 = s - g2 * G3;
        const float* p = td.w + static_cast<u64>(g2) * b2 * d3 + static_cast<u64>(g3) * (4u * Q);
        for (u32 r0 = 0; r0 < b2; r0 += G) {
            float4 v[G][Q];
#pragma unroll
            for (int g = 0; g < G; ++g)
#pragma unroll
                for (int q = 0; q < Q; ++q)
                    if (r0 + g < b2) {
                        const float* src = p + static_cast<u64>(r0 + g) * d3 + q * 4;
                        v[g][q] = (Q == 1) ? ld4_stream(src) : *reinterpret_cast<const float4*>(src);
                    }
#pragma unroll
            for (int g = 0; g < G; ++g)
                if (r0 + g < b2) {
#pragma unroll
                    for (int q = 0; q < Q; ++q) acc = add_squares(acc, v[g][q]);
                }
        }
    }
    a.keys[u] = static_cast<u64>(__double_as_longlong(acc)) & 0x7FFFFFFFFFFFFFFFull;
    if (sumsq) sumsq[u] = acc;
    if (norms) norms[u] = static_cast<float>(sqrt(acc));
}

// Row structures (filters, neurons: structure s of a tensor is the contiguous run [s L, (s+1) L) of its
// memory): thread-per-structure loads would touch one cache line per lane, so the workgroup stages
// 32-element pieces of its 256 rows through LDS with coalesced 128-bit loads (8 lanes per row piece) and
// every thread then adds its own row's piece in memory order -- the same additions in the same order as
// k_struct_sumsq.  Rows are padded to 33 words so that the per-thread reads hit distinct banks.
constexpr int kRowTile = 32;

__global__ __launch_bounds__(kBlock) void k_struct_sumsq_rows(StructArgs a, double* sumsq, float* norms) {
    __shared__ float s_tile[kBlock][kRowTile + 1];
    __shared__ const float* s_row[kBlock];
    __shared__ u32 s_len[kBlock];
    __shared__ u32 s_maxlen, s_minlen, s_aligned;
    const int tid = threadIdx.x;
    const u64 u = static_cast<u64>(blockIdx.x) * kBlock + tid;
    if (tid == 0) { s_maxlen = 0; s_minlen = 0xFFFFFFFFu; s_aligned = 1; }
    __syncthreads();
    u32 len = 0;
    const float* row = nullptr;
    if (u < a.F) {
        const int t = tensor_of_struct(a.td, a.n_tensors, u);
        const TensorDesc& td = a.td[t];
        len = td.d[3];
        row = td.w + (u - td.struct_start) * len;
    }
    s_row[tid] = row;
    s_len[tid] = len;
    atomicMax(&s_maxlen, len);
    atomicMin(&s_minlen, len);                            // 0 when the last workgroup is ragged
    if (row && (reinterpret_cast<uintptr_t>(row) & 15u)) atomicAnd(&s_aligned, 0u);
    __syncthreads();
    const u32 maxlen = s_maxlen;
    const u32 fast_end = s_aligned ? (s_minlen / kRowTile) * kRowTile : 0;   // pieces below it: unguarded loads
    const int seg = tid & 7, sub = tid >> 3;              // 8 lanes per row piece, 32 rows per pass
    double acc = 0.0;
    // Pieces below fast_end are fetched one iteration ahead, so that the loads of piece i+1 are in flight
    // while piece i is added up.
    float4 v[8];
    if (fast_end > 0) {
#pragma unroll
        for (int pass = 0; pass < 8; ++pass) v[pass] = ld4_stream(s_row[pass * 32 + sub] + seg * 4);
    }
    for (u32 cb = 0; cb < maxlen; cb += kRowTile) {
        if (cb < fast_end) {
#pragma unroll
            for (int pass = 0; pass < 8; ++pass) {
                float* dst = &s_tile[pass * 32 + sub][seg * 4];
                dst[0] = v[pass].x; dst[1] = v[pass].y; dst[2] = v[pass].z; dst[3] = v[pass].w;
            }
            if (cb + kRowTile < fast_end) {
#pragma unroll
                for (int pass = 0; pass < 8; ++pass)
                    v[pass] = ld4_stream(s_row[pass * 32 + sub] + cb + kRowTile + seg * 4);
            }
        } else {
            for (int pass = 0; pass < 8; ++pass) {
                const int st = pass * 32 + sub;
                const u32 L = s_len[st];
                const float* p = s_row[st];
                float* dst = &s_tile[st][seg * 4];
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const u32 x = cb + seg * 4 + k;
                    dst[k] = (x < L) ? p[x] : 0.0f;
                }
            }
        }
        __syncthreads();
        if (len > cb) {
            const u32 m = (len - cb < static_cast<u32>(kRowTile)) ? len - cb : static_cast<u32>(kRowTile);
            if (m == kRowTile) {
#pragma unroll
                for (int j = 0; j < kRowTile; ++j) {
                    const double x = static_cast<double>(s_tile[tid][j]);
                    acc = acc + x * x;
                }
            } else {
                for (u32 j = 0; j < m; ++j) {
                    const double x = static_cast<double>(s_tile[tid][j]);
                    acc = acc + x * x;
                }
            }
        }
        __syncthreads();
    }
    if (u < a.F) {
        a.keys[u] = static_cast<u64>(__double_as_longlong(acc)) & 0x7FFFFFFFFFFFFFFFull;
        if (sumsq) sumsq[u] = acc;
        if (norms) norms[u] = static_cast<float>(sqrt(acc));
    }
}

// The same aggregation for calls with few row structures (a CIFAR ResNet's 2 032 filters, a VGG's 5 504):
// 256 rows per workgroup would leave most of the chip idle and every 32-element piece costs a load
// latency, so here a workgroup takes kFewRows rows and stages kFewTile elements of each per step: one
// wavefront fetches one row's piece per load instruction (1 KB contiguous), eight loads per thread are in
// flight, the next piece is requested before the current one is added up, and the first kFewRows threads
// add their rows' pieces in memory order.  Rows of any length and alignment: a float4 that lies inside
// an aligned row is one 128-bit load, anything else is fetched element by element.
constexpr int kFewRows = 32;
constexpr int kFewTile = 256;

__global__ __launch_bounds__(kBlock) void k_struct_sumsq_rows_few(StructArgs a, double* sumsq, float* norms) {
    __shared__ float s_tile[kFewRows][kFewTile + 1];
    __shared__ const float* s_row[kFewRows];
    __shared__ u32 s_len[kFewRows];
    __shared__ u32 s_vec[kFewRows];
    __shared__ u32 s_maxlen;
    const int tid = threadIdx.x;
    const u64 u = static_cast<u64>(blockIdx.x) * kFewRows + tid;          // the row of thread tid < kFewRows
    if (tid == 0) s_maxlen = 0;
    __syncthreads();
    u32 len = 0;
    if (tid < kFewRows) {
        const float* row = nullptr;
        if (u < a.F) {
            const int t = tensor_of_struct(a.td, a.n_tensors, u);
            const TensorDesc& td = a.td[t];
            len = td.d[3];
            row = td.w + (u - td.struct_start) * len;
        }
        s_row[tid] = row;
        s_len[tid] = len;
        s_vec[tid] = (row && (reinterpret_cast<uintptr_t>(row) & 15u) == 0) ? 1u : 0u;
        atomicMax(&s_maxlen, len);
    }
    __syncthreads();
    const u32 maxlen = s_maxlen;
    const int col = (tid & 63) * 4, wave = tid >> 6;                      // wavefront `wave` fetches rows 4 p + wave
    float4 v[8];
    auto fetch = [&](u32 cb) {
#pragma unroll
        for (int p = 0; p < 8; ++p) {
            const int st = p * 4 + wave;
            const u32 L = s_len[st];
            const u32 x = cb + col;
            const float* src = s_row[st];
            float4 t = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
            if (x + 4 <= L && s_vec[st]) {
                t = *reinterpret_cast<const float4*>(src + x);
            } else if (x < L) {
                t.x = src[x];
                if (x + 1 < L) t.y = src[x + 1];
                if (x + 2 < L) t.z = src[x + 2];
                if (x + 3 < L) t.w = src[x + 3];
            }
            v[p] = t;
        }
    };
    double acc = 0.0;
    if (maxlen > 0) fetch(0);
    for (u32 cb = 0; cb < maxlen; cb += kFewTile) {
#pragma unroll
        for (int p = 0; p < 8; ++p) {
            float* dst = &s_tile[p * 4 + wave][col];
            dst[0] = v[p].x; dst[1] = v[p].y; dst[2] = v[p].z; dst[3] = v[p].w;
        }
        if (cb + kFewTile < maxlen) fetch(cb + kFewTile);
        __syncthreads();
        if (tid < kFewRows && len > cb) {
            const u32 m = (len - cb < static_cast<u32>(kFewTile)) ? len - cb : static_cast<u32>(kFewTile);
            u32 j = 0;
            for (; j + 16 <= m; j += 16) {                // sixteen LDS reads at a time ahead of the addition chain
                float t[16];
#pragma unroll
                for (int k = 0; k < 16; ++k) t[k] = s_tile[tid][j + k];
#pragma unroll
                for (int k = 0; k < 16; ++k) {
                    const double x = static_cast<double>(t[k]);
                    acc = acc + x * x;
                }
            }
            for (; j < m; ++j) {
                const double x = static_cast<double>(s_tile[tid][j]);
                acc = acc + x * x;
            }
        }
        __syncthreads();
    }
    if (tid < kFewRows && u < a.F) {
        a.keys[u] = static_cast<u64>(__double_as_longlong(acc)) & 0x7FFFFFFFFFFFFFFFull;
        if (sumsq) sumsq[u] = acc;
        if (norms) norms[u] = static_cast<float>(sqrt(acc));
    }
}

// Histogram of one radix level over the aggregate keys (one ranking per group).  Measured on 18.9 M keys: the
// first levels take 50-65 us and the last ones 31 us because the keys come from HBM the first time and from the
// last-level cache afterwards; 1024-thread workgroups (fewer flushes) and adding a wavefront's equal digits with
// one LDS atomic changed nothing at the upper levels and cost 7 us at the lower ones.
__global__ __launch_bounds__(kBlock) void k_hist_keys(StructArgs a, int level, u64 chunks_per_block) {
    __shared__ u32 s_hist[kBins];
    __shared__ u64 s_prefix;
    __shared__ u32 s_active;
    __shared__ u64 s_mprefix;             // merged form: the ranking's state on entering this level
    __shared__ u32 s_mactive;
    if (a.only_failed && a.ctl->window_failed == 0) return;
    const u64 c0 = static_cast<u64>(blockIdx.x) * chunks_per_block;
    if (c0 >= a.n_schunks) return;
    const u64 c1 = (c0 + chunks_per_block < a.n_schunks) ? c0 + chunks_per_block : a.n_schunks;
    const Level L = level_of(63, level);
    const int nb = 1 << L.bits;
    const int tid = threadIdx.x;
    if (a.merged) {                       // every workgroup derives the same state, workgroup 0 stores it
        if (tid < 64) {
            const SlotStep e = (level == 0) ? slot_canonical(a.slots[0])
                                            : wave_enter_level(a.slots[0], level, 63, struct_hist(a, level - 1), struct_coarse(a, level - 1));
            if (tid == 0) {
                s_mprefix = e.prefix;
                s_mactive = (e.state == kSelecting) ? 1u : 0u;
                if (blockIdx.x == 0 && level > 0) a.slots[0].step[level & 1] = e;
            }
        }
        __syncthreads();
    }
    auto flush = [&](long long group) {
        u64* dst = a.merged ? struct_hist(a, level) : a.histx + static_cast<u64>(group) * kBins;
        for (int i = tid; i < nb; i += kBlock) {
            const u32 v = s_hist[i];
            if (v) atomicAdd(reinterpret_cast<unsigned long long*>(dst + i), static_cast<unsigned long long>(v));
        }
        if (a.merged && tid < kCoarse) {  // the coarse sums of the same counts
            const int run = coarse_run(nb);
            u32 v = 0;
            for (int t = tid * run; t < (tid + 1) * run && t < nb; ++t) v += s_hist[t];
            if (v) atomicAdd(reinterpret_cast<unsigned long long*>(struct_coarse(a, level) + tid), static_cast<unsigned long long>(v));
        }
    };
    long long cur_group = -1;
    for (u64 c = c0; c < c1; ++c) {
        const int t = tensor_of_schunk(a.td, a.n_tensors, c);
        const long long g = a.per_tensor ? t : 0;
        if (g != cur_group) {
            if (cur_group >= 0) {
                __syncthreads();
                flush(cur_group);
            }
            __syncthreads();
            if (tid == 0 && a.merged) {
                s_prefix = s_mprefix;
                s_active = s_mactive;
            } else if (tid == 0) {
                const Slot& s = a.slots[g];
                s_prefix = s.prefix;
                s_active = (s.state == kSelecting) ? 1u : 0u;
            }
            for (int i = tid; i < nb; i += kBlock) s_hist[i] = 0;
            __syncthreads();
            cur_group = g;
        }
        if (!s_active) continue;
        const TensorDesc& td = a.td[t];
        const u64 base = (c - td.pad) * kChunk;
        const u64 prefix = s_prefix;
        const u64 end = (base + kChunk < td.n_struct) ? base + kChunk : td.n_struct;
        const u64* __restrict__ kp = a.keys + td.struct_start;
        // eight keys per step so that their loads overlap (a chunk is 32 keys per thread)
        for (u64 i0 = base + tid; i0 < end; i0 += 8 * kBlock) {
            u64 key[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const u64 i = i0 + static_cast<u64>(u) * kBlock;
                key[u] = (i < end) ? kp[i] : ~prefix;      // a filler that fails the prefix test at every level
            }
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (i0 + static_cast<u64>(u) * kBlock < end && ((key[u] ^ prefix) >> L.hi_shift) == 0)
                    atomicAdd(&s_hist[(key[u] >> L.shift) & (nb - 1)], 1u);
        }
    }
    if (cur_group >= 0) {
        __syncthreads();
        flush(cur_group);
    }
}

__global__ __launch_bounds__(kBlock) void k_tie_count_keys(StructArgs a) {
    __shared__ u32 s_cnt;
    __shared__ SlotStep s_e;
    const u64 c = blockIdx.x;
    if (c >= a.n_schunks) return;
    const int tid = threadIdx.x;
    u64 T;
    const int t = tensor_of_schunk(a.td, a.n_tensors, c);
    if (a.merged) {                       // the last level is folded in here; k_tie_locate_keys stores the outcome
        if (tid < 64) {
            const int last = n_levels(63) - 1;
            const SlotStep e = wave_enter_level(a.slots[0], last + 1, 63, struct_hist(a, last), struct_coarse(a, last));
            if (tid == 0) s_e = e;
        }
        __syncthreads();
        if (!(s_e.state == kDone && s_e.need_tie)) return;
        T = s_e.prefix;
    } else {
        if (a.ctl->need_tie == 0) return;
        const u64 g = a.per_tensor ? t : 0;
        const Slot& s = a.slots[g];
        if (!(s.state == kDone && s.need_tie)) return;
        T = s.prefix;
    }
    if (tid == 0) s_cnt = 0;
    __syncthreads();
    const TensorDesc& td = a.td[t];
    const u64 base = (c - td.pad) * kChunk;
    u32 mine = 0;
    for (u64 i = base + tid; i < base + kChunk && i < td.n_struct; i += kBlock)
        mine += (a.keys[td.struct_start + i] == T) ? 1u : 0u;
    if (mine) atomicAdd(&s_cnt, mine);
    __syncthreads();
    if (tid == 0) a.tiecnt[c] = s_cnt;
}

// One workgroup per ranking: index search among tied aggregates, then the public record.
__global__ __launch_bounds__(kBlock) void k_tie_locate_keys(StructArgs a, condensa_select* results) {
    __shared__ u64 s_wave[kBlock / 64];
    __shared__ u64 s_found[3];
    __shared__ SlotStep s_e;
    const int g = blockIdx.x;
    const int tid = threadIdx.x;
    Slot& slot = a.slots[g];
    if (a.merged) {
        // the last level's histogram is folded in here, and this workgroup (the only one that touches the
        // ranking in this kernel) makes the outcome the ranking's stored state
        if (tid < 64) {
            const int last = n_levels(63) - 1;
            const SlotStep e = wave_enter_level(slot, last + 1, 63, struct_hist(a, last), struct_coarse(a, last));
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
    if (need) {
        const u64 r = s_e.remaining;
        const u64 T = s_e.prefix;
        const u64 cb = a.per_tensor ? a.td[g].pad : 0;
        const u64 ce = a.per_tensor ? a.td[g + 1].pad : a.n_schunks;
        const u64 per = (ce - cb + kBlock - 1) / kBlock;
        const u64 my0 = cb + per * tid < ce ? cb + per * tid : ce;
        const u64 my1 = my0 + per < ce ? my0 + per : ce;
        u64 mine = 0;
        for (u64 c = my0; c < my1; ++c) mine += a.tiecnt[c];
        u64 total;
        const u64 before = block_excl_scan_u64(mine, s_wave, &total);
        if (tid == 0) s_found[2] = 0;
        __syncthreads();
        if (before < r && r <= before + mine) {
            u64 cum = before;
            for (u64 c = my0; c < my1; ++c) {
                const u64 x = a.tiecnt[c];
                if (r <= cum + x) { s_found[0] = c; s_found[1] = r - cum; s_found[2] = 1; break; }
                cum += x;
            }
        }
        __syncthreads();
        if (s_found[2]) {
            const u64 c = s_found[0];
            const u64 rr = s_found[1];
            const int t = tensor_of_schunk(a.td, a.n_tensors, c);
            const TensorDesc& td = a.td[t];
            const u64 base = (c - td.pad) * kChunk;
            constexpr int kRun = kChunk / kBlock;
            const u64 i_begin = base + static_cast<u64>(tid) * kRun;
            u32 hits = 0;
            for (int k = 0; k < kRun; ++k) {
                const u64 i = i_begin + k;
                if (i >= td.n_struct) break;
                hits += (a.keys[td.struct_start + i] == T) ? 1u : 0u;
            }
            u64 tot2;
            const u64 bef2 = block_excl_scan_u64(hits, s_wave, &tot2);
            if (bef2 < rr && rr <= bef2 + hits) {
                u64 seen = bef2;
                for (int k = 0; k < kRun; ++k) {
                    const u64 i = i_begin + k;
                    if (i >= td.n_struct) break;
                    if (a.keys[td.struct_start + i] == T) {
                        ++seen;
                        if (seen == rr) { slot.tie_end = (a.per_tensor ? 0 : td.struct_start) + i + 1; break; }
                    }
                }
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
        } else {
            out.n_gt = 0; out.n_tie_kept = 0; out.n_tie = 0;
            out.threshold_key = ~static_cast<u64>(0);
            out.tie_end = 0;
        }
        out.path = slot.path;
        results[g] = out;
    }
}

// ---- small groups: ranking, tie rule, structure mask and kept-id list in one workgroup ----------------
//
// A CIFAR ResNet has 2 032 filters, its layers 16 to 64 each: rankings of that size are
// bound by launch latency (six histogram + scan launch pairs, tie kernels, mask, scan, compaction: 19
// launches of ~4.5 us).  One workgroup of 1024 threads per group does the same steps back to back: six
// radix levels with an LDS histogram, the index search among tied aggregates, keep flags and the ordered
// list of kept ids (every thread owns a contiguous run of structures, so a workgroup scan orders them).
// Used when no group has more than kSmallGroup structures.

constexpr int kSmallThreads = 1024;
constexpr u64 kSmallGroup = 4096;       // measured: 2 032 filters 0.141 -> 0.100 ms per call, 43 008 blocks 0.22 -> 0.30 ms

// Exclusive scan over the 1024 threads of the workgroup in thread order; *total gets the sum.
// s_part holds kSmallThreads / 64 entries.  All threads must call it.
__device__ inline u64 small_excl_scan(u64 v, u64* s_part, u64* total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const u64 incl = wave_incl_scan_u64(v);
    __syncthreads();                                       // s_part may still be read from a previous call
    if (lane == 63) s_part[wave] = incl;
    __syncthreads();
    u64 before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < kSmallThreads / 64; ++w) {
        const u64 t = s_part[w];
        if (w < wave) before += t;
        all += t;
    }
    *total = all;
    return before + incl - v;
}

__global__ __launch_bounds__(kSmallThreads) void k_struct_small(StructArgs a, u8* user_mask, int32_t* keep_idx,
                                                                condensa_select* results) {
    __shared__ u32 s_hist[kBins];
    __shared__ u64 s_part[kSmallThreads / 64];
    __shared__ u64 s_sel[3];                               // bin, rank inside it, entries in it
    __shared__ u64 s_tie_end;
    const int g = blockIdx.x;
    const int tid = threadIdx.x;
    Slot& slot = a.slots[g];
    const u64 first = a.per_tensor ? a.td[g].struct_start : 0;
    const u64 n = a.per_tensor ? a.td[g + 1].struct_start - first : a.F;
    const u64 k = slot.k;
    const u64* __restrict__ keys = a.keys + first;

    // kept structures of the groups before this one: their kept counts are fixed by the density
    u64 kept_before = 0;
    if (keep_idx && g > 0) {
        u64 part = 0;
        for (int i = tid; i < g; i += kSmallThreads) part += a.slots[i].k;
        u64 tot;
        small_excl_scan(part, s_part, &tot);
        kept_before = tot;
    }

    u64 T = ~static_cast<u64>(0), keep_ties = 0, n_tie = 0, tie_end = 0;
    if (k > 0) {                                           // uniform over the workgroup
        u64 prefix = 0, remaining = k;
        for (int level = 0; level < n_levels(63); ++level) {
            const Level L = level_of(63, level);
            const int nb = 1 << L.bits;
            for (int i = tid; i < nb; i += kSmallThreads) s_hist[i] = 0;
            __syncthreads();
            for (u64 i = tid; i < n; i += kSmallThreads) {
                const u64 key = keys[i];
                if (((key ^ prefix) >> L.hi_shift) == 0) atomicAdd(&s_hist[(key >> L.shift) & (nb - 1)], 1u);
            }
            __syncthreads();
            // two bins per thread, from the top
            u64 cnt[2], sum = 0;
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int b = nb - 1 - (tid * 2 + j);
                cnt[j] = (b >= 0) ? s_hist[b] : 0;
                sum += cnt[j];
            }
            u64 total;
            u64 cum = small_excl_scan(sum, s_part, &total);
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int b = nb - 1 - (tid * 2 + j);
                if (b >= 0 && cum < remaining && remaining <= cum + cnt[j]) {
                    s_sel[0] = static_cast<u64>(b);
                    s_sel[1] = remaining - cum;
                    s_sel[2] = cnt[j];
                }
                cum += cnt[j];
            }
            __syncthreads();                               // k <= n, so exactly one thread wrote s_sel
            prefix |= s_sel[0] << L.shift;
            remaining = s_sel[1];
            n_tie = s_sel[2];
            __syncthreads();
        }
        T = prefix;
        keep_ties = remaining;
    }

    // every thread owns the contiguous run [i0, i1) of the group
    const u64 per = (n + kSmallThreads - 1) / kSmallThreads;
    const u64 i0 = per * tid < n ? per * tid : n;
    const u64 i1 = i0 + per < n ? i0 + per : n;
    if (k > 0) {
        tie_end = n;
        if (keep_ties < n_tie) {                           // uniform: find the keep_ties-th tie in index order
            u64 mine = 0;
            for (u64 i = i0; i < i1; ++i) mine += (keys[i] == T) ? 1u : 0u;
            u64 total;
            const u64 before = small_excl_scan(mine, s_part, &total);
            if (before < keep_ties && keep_ties <= before + mine) {
                u64 seen = before;
                for (u64 i = i0; i < i1; ++i) {
                    if (keys[i] == T && ++seen == keep_ties) { s_tie_end = i + 1; break; }
                }
            }
            __syncthreads();
            tie_end = s_tie_end;
        }
    }
    // keep flags and the ordered list of kept ids
    u64 kept = 0;
    for (u64 i = i0; i < i1; ++i) {
        const u64 key = keys[i];
        const u32 keep = (k > 0 && (key > T || (key == T && i < tie_end))) ? 1u : 0u;
        a.smask[first + i] = static_cast<u8>(keep);
        if (user_mask) user_mask[first + i] = static_cast<u8>(keep);
        kept += keep;
    }
    if (keep_idx) {
        u64 total;
        u64 pos = kept_before + small_excl_scan(kept, s_part, &total);
        for (u64 i = i0; i < i1; ++i)
            if (a.smask[first + i]) keep_idx[pos++] = static_cast<int32_t>(first + i);
    }
    if (tid == 0) {
        condensa_select out;
        out.n = slot.n;
        out.k = k;
        out.n_gt = k > 0 ? k - keep_ties : 0;
        out.n_tie_kept = keep_ties;
        out.n_tie = n_tie;
        out.threshold_key = T;
        out.tie_end = tie_end;
        out.path = slot.path;
        results[g] = out;
    }
}

// Structures per thread and per workgroup of the mask / kept-index passes.
constexpr int kMaskPer = 4;
constexpr int kMaskTile = kBlock * kMaskPer;
constexpr int kScanThreads = 1024;

// inclusive scan of one u32 per thread over the workgroup; *total = workgroup sum.  Ends with a barrier.
template <int THREADS>
__device__ inline u32 wg_incl_scan_u32(u32 v, u32* s_wave, u32* total) {
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    u32 inc = v;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const u32 o = __shfl_up(inc, off);
        if (lane >= off) inc += o;
    }
    if (lane == 63) s_wave[wv] = inc;
    __syncthreads();
    u32 before = 0, tot = 0;
#pragma unroll
    for (int j = 0; j < THREADS / 64; ++j) {
        const u32 x = s_wave[j];
        if (j < wv) before += x;
        tot += x;
    }
    __syncthreads();
    *total = tot;
    return before + inc;
}

// keep flag of every structure and the number of kept structures of every tile of kMaskTile.
// The one-sweep form of block pruning (k_struct_fused.h) leaves the flags in `smask` itself: its sweep decides
// every block outside the window, its fix-up the listed ones.  There kMaskFromFlags only counts and copies
// them (18.9 MB instead of 151 MB of keys), and kMaskIfFailed derives them from the keys when the window failed.
enum : int { kMaskFromKeys = 0, kMaskFromFlags = 1, kMaskIfFailed = 2 };
__global__ __launch_bounds__(kBlock) void k_struct_mask(StructArgs a, u8* user_mask, int mode) {
    __shared__ u32 s_wave[kBlock / 64];
    if (mode == kMaskFromFlags && a.ctl->window_failed != 0) return;
    if (mode == kMaskIfFailed && a.ctl->window_failed == 0) return;
    const int tid = threadIdx.x;
    const u64 u0 = (static_cast<u64>(blockIdx.x) * kBlock + tid) * kMaskPer;
    u32 keep[kMaskPer] = {0, 0, 0, 0};
    if (u0 < a.F && mode == kMaskFromFlags) {
        const bool full = u0 + kMaskPer <= a.F;
        if (full) {
            const uchar4 m4 = *reinterpret_cast<const uchar4*>(a.smask + u0);
            keep[0] = m4.x; keep[1] = m4.y; keep[2] = m4.z; keep[3] = m4.w;
            if (user_mask) {
                if ((reinterpret_cast<uintptr_t>(user_mask) & 3u) == 0) *reinterpret_cast<uchar4*>(user_mask + u0) = m4;
                else for (int k = 0; k < kMaskPer; ++k) user_mask[u0 + k] = static_cast<u8>(keep[k]);
            }
        } else {
            for (int k = 0; k < kMaskPer; ++k)
                if (u0 + k < a.F) {
                    keep[k] = a.smask[u0 + k];
                    if (user_mask) user_mask[u0 + k] = static_cast<u8>(keep[k]);
                }
        }
    } else if (u0 < a.F) {
        const bool full = u0 + kMaskPer <= a.F;
        u64 key[kMaskPer] = {0, 0, 0, 0};
        if (full) {
            const ulonglong2 k01 = *reinterpret_cast<const ulonglong2*>(a.keys + u0);
            const ulonglong2 k23 = *reinterpret_cast<const ulonglong2*>(a.keys + u0 + 2);
            key[0] = k01.x; key[1] = k01.y; key[2] = k23.x; key[3] = k23.y;
        } else {
            for (int k = 0; k < kMaskPer; ++k) if (u0 + k < a.F) key[k] = a.keys[u0 + k];
        }
        int t = a.per_tensor ? tensor_of_struct(a.td, a.n_tensors, u0) : 0;
#pragma unroll
        for (int k = 0; k < kMaskPer; ++k) {
            const u64 u = u0 + k;
            if (u >= a.F) break;
            u64 idx = u;
            if (a.per_tensor) {
                while (t + 1 < a.n_tensors && a.td[t + 1].struct_start <= u) ++t;
                idx = u - a.td[t].struct_start;
            }
            const Slot& s = a.slots[a.per_tensor ? t : 0];
            keep[k] = (key[k] > s.prefix || (key[k] == s.prefix && idx < s.tie_end)) ? 1u : 0u;
            if (s.state == kInactive) keep[k] = 0;
        }
        const uchar4 m4 = make_uchar4(static_cast<u8>(keep[0]), static_cast<u8>(keep[1]), static_cast<u8>(keep[2]),
                                      static_cast<u8>(keep[3]));
        if (full) {
            *reinterpret_cast<uchar4*>(a.smask + u0) = m4;
            if (user_mask) {
                if ((reinterpret_cast<uintptr_t>(user_mask) & 3u) == 0) *reinterpret_cast<uchar4*>(user_mask + u0) = m4;
                else for (int k = 0; k < kMaskPer; ++k) user_mask[u0 + k] = static_cast<u8>(keep[k]);
            }
        } else {
            for (int k = 0; k < kMaskPer; ++k)
                if (u0 + k < a.F) {
                    a.smask[u0 + k] = static_cast<u8>(keep[k]);
                    if (user_mask) user_mask[u0 + k] = static_cast<u8>(keep[k]);
                }
        }
    }
    u32 total;
    wg_incl_scan_u32<kBlock>(keep[0] + keep[1] + keep[2] + keep[3], s_wave, &total);
    if (tid == 0) a.sblock[blockIdx.x] = total;
}

// exclusive scan of the per-tile counts (single workgroup, 4 counts per thread and step)
__global__ __launch_bounds__(kScanThreads) void k_struct_scan_blocks(u32* sblock, u64 n_blocks) {
    __shared__ u32 s_wave[kScanThreads / 64];
    u32 running = 0;
    for (u64 base = 0; base < n_blocks; base += kScanThreads * 4) {
        const u64 i = base + static_cast<u64>(threadIdx.x) * 4;
        u32 v[4] = {0, 0, 0, 0};
        const bool full = i + 4 <= n_blocks;
        if (full) {
            const uint4 x = *reinterpret_cast<const uint4*>(sblock + i);
            v[0] = x.x; v[1] = x.y; v[2] = x.z; v[3] = x.w;
        } else {
            for (int k = 0; k < 4; ++k) if (i + k < n_blocks) v[k] = sblock[i + k];
        }
        const u32 sum = v[0] + v[1] + v[2] + v[3];
        u32 total;
        const u32 ex = running + wg_incl_scan_u32<kScanThreads>(sum, s_wave, &total) - sum;
        if (full) {
            *reinterpret_cast<uint4*>(sblock + i) = make_uint4(ex, ex + v[0], ex + v[0] + v[1], ex + v[0] + v[1] + v[2]);
        } else {
            u32 e = ex;
            for (int k = 0; k < 4; ++k) if (i + k < n_blocks) { sblock[i + k] = e; e += v[k]; }
        }
        running += total;
    }
}

// ascending ids of the kept structures
__global__ __launch_bounds__(kBlock) void k_struct_keep_idx(StructArgs a, int32_t* keep_idx) {
    __shared__ u32 s_wave[kBlock / 64];
    const u64 u0 = (static_cast<u64>(blockIdx.x) * kBlock + threadIdx.x) * kMaskPer;
    u32 m[kMaskPer] = {0, 0, 0, 0};
    if (u0 + kMaskPer <= a.F) {
        const uchar4 x = *reinterpret_cast<const uchar4*>(a.smask + u0);
        m[0] = x.x; m[1] = x.y; m[2] = x.z; m[3] = x.w;
    } else {
        for (int k = 0; k < kMaskPer; ++k) if (u0 + k < a.F) m[k] = a.smask[u0 + k];
    }
    const u32 sum = m[0] + m[1] + m[2] + m[3];
    u32 total;
    u64 pos = static_cast<u64>(a.sblock[blockIdx.x]) + wg_incl_scan_u32<kBlock>(sum, s_wave, &total) - sum;
#pragma unroll
    for (int k = 0; k < kMaskPer; ++k)
        if (m[k]) keep_idx[pos++] = static_cast<int32_t>(u0 + k);
}

// theta = w on kept structures, +0 elsewhere; element mask = structure mask broadcast
template <bool VEC>
__device__ inline void struct_apply_tile(const StructArgs& a, const OutDesc* __restrict__ out, u64 tile) {
    const u64 c = tile / kSubPerChunk;
    const u32 sub = static_cast<u32>(tile % kSubPerChunk);
    if (c >= a.n_chunks) return;
    const int tid = threadIdx.x;
    const int t = static_cast<int>(a.chunk_map[c]);
    const TensorDesc& td = a.td[t];
    const u64 n = td.n;
    const u64 wg0 = (c - td.chunk_start) * kChunk + static_cast<u64>(sub) * (kBlock * 4);
    if (wg0 >= n) return;                                                // uniform
    const u64 e0 = wg0 + tid * 4;
    const bool full = VEC && wg0 + kBlock * 4 <= n;                      // uniform: unguarded 128-bit accesses
    if (!full && e0 >= n) return;
    const OutDesc o = out[t];
    const u8* __restrict__ sm = a.smask + td.struct_start;
    const u32 d1 = td.d[1], d2 = td.d[2], d3 = td.d[3];
    const u32 b0 = td.b[0], b1 = td.b[1], b2 = td.b[2], b3 = td.b[3];
    const u32 G1 = fast_div(d1 + b1 - 1, td.fd[kDivB1]), G2 = fast_div(d2 + b2 - 1, td.fd[kDivB2]),
              G3 = fast_div(d3 + b3 - 1, td.fd[kDivB3]);
    float v[4];
    if (full) {
        const float4 x = ld4_stream(td.w + e0);
        v[0] = x.x; v[1] = x.y; v[2] = x.z; v[3] = x.w;
    } else {
        load4<VEC>(td.w, e0, n, v);
    }
    // Coordinates of the first element; the others follow by carrying along the last dimension.  Below
    // 2^32 elements every quotient comes from the host's reciprocals (a hardware-free u32 division costs
    // ~30 instructions, and a dozen of them per thread made this sweep ALU-bound).
    const bool small = n <= 0xFFFFFFFFull;
    u64 r;
    u32 x3;
    if (small) {
        const u32 e32 = static_cast<u32>(e0);
        const u32 q = fast_div(e32, td.fd[kDivD3]);
        r = q;
        x3 = e32 - q * d3;
    } else {
        r = e0 / d3;
        x3 = static_cast<u32>(e0 % d3);
    }
    auto row_base = [&](u64 row) -> u64 {               // structure id of column block 0 in this row
        if (small) {
            const u32 r32 = static_cast<u32>(row);
            const u32 q = fast_div(r32, td.fd[kDivD2]);
            const u32 x2 = r32 - q * d2;
            const u32 x0 = fast_div(q, td.fd[kDivD1]);
            const u32 x1 = q - x0 * d1;
            return ((static_cast<u64>(fast_div(x0, td.fd[kDivB0])) * G1 + fast_div(x1, td.fd[kDivB1])) * G2 +
                    fast_div(x2, td.fd[kDivB2])) * G3;
        }
        const u64 x2 = row % d2;
        const u64 q = row / d2;
        const u64 x1 = q % d1;
        const u64 x0 = q / d1;
        return (((x0 / b0) * G1 + x1 / b1) * G2 + x2 / b2) * G3;
    };
    u64 gbase = row_base(r);
    u32 cb = fast_div(x3, td.fd[kDivB3]);               // column block and position inside it
    u32 xin = x3 - cb * b3;
    float th[4];
    u8 m[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        if (x3 >= d3) { x3 = 0; cb = 0; xin = 0; ++r; gbase = row_base(r); }
        u8 keep = 0;
        if (full || e0 + k < n) keep = sm[gbase + cb];
        m[k] = keep;
        th[k] = keep ? v[k] : 0.0f;
        ++x3;
        if (++xin == b3) { xin = 0; ++cb; }
    }
    if (full) {
        if (o.theta) st4_stream(o.theta + e0, th[0], th[1], th[2], th[3]);
        if (o.mask) st_mask4_stream(o.mask + e0, m[0], m[1], m[2], m[3]);
    } else {
        if (o.theta) store4<VEC>(o.theta, e0, n, th);
        if (o.mask) store4_u8<VEC>(o.mask, e0, n, m);
    }
}

template <bool VEC>
__global__ __launch_bounds__(kBlock) void k_struct_apply(StructArgs a, const OutDesc* __restrict__ out) {
    struct_apply_tile<VEC>(a, out, blockIdx.x);
}

// Thinning gather: out[o', i', r] = w[keep_out[o'] - off_out, keep_in[i'] - off_in, r]; NULL list = identity.
// An id outside the tensor writes +0 instead of reading out of bounds.
__global__ __launch_bounds__(kBlock) void k_thin(const float* __restrict__ w, u64 c_out, u64 c_in, u64 ksize,
                                                 const int32_t* __restrict__ keep_out, u64 n_out, int64_t off_out,
                                                 const int32_t* __restrict__ keep_in, u64 n_in, int64_t off_in,
                                                 float* __restrict__ out) {
    const u64 total = n_out * n_in * ksize;
    const u64 stride = static_cast<u64>(gridDim.x) * kBlock;
    const u64 per_out = n_in * ksize;
    for (u64 i = static_cast<u64>(blockIdx.x) * kBlock + threadIdx.x; i < total; i += stride) {
        const u64 o = i / per_out;
        const u64 rem = i - o * per_out;
        const u64 ic = rem / ksize;
        const u64 r = rem - ic * ksize;
        const int64_t so = keep_out ? static_cast<int64_t>(keep_out[o]) - off_out : static_cast<int64_t>(o);
        const int64_t si = keep_in ? static_cast<int64_t>(keep_in[ic]) - off_in : static_cast<int64_t>(ic);
        float v = 0.0f;
        if (so >= 0 && static_cast<u64>(so) < c_out && si >= 0 && static_cast<u64>(si) < c_in)
            v = w[(static_cast<u64>(so) * c_in + static_cast<u64>(si)) * ksize + r];
        out[i] = v;
    }
}

}  // namespace condensa
