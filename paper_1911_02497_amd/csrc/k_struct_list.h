// Structure rankings of moderate size (more than k_struct_small's 4096 structures, at most kSmallCallElems, GLOBAL
// scope): two radix levels over the aggregates, then a list.
//
// The six levels of a 63-bit ranking are six dependent launches plus the tie search.  Aggregates of one model share
// their sign and most exponent bits, so level 0 barely separates them; after level 1 (22 of 63 bits) the threshold's
// bin holds a few hundred structures.  k_struct_list_collect lists those (key, structure id) pairs and
// k_struct_list_finish, one workgroup, finishes on the list as k_small_finish does for element pruning: the four
// remaining levels in LDS, the lowest-id rule among equal aggregates, the stored state and the record.  The list
// can hold every structure, so nothing overflows.  A Transformer's 688 128 blocks of 8x8: 14 -> 10 launches.
// Table 1 (FilterPrune, BlockPrune: structures are aggregated and pruned); Section 3.1.
#pragma once
#include "k_small.h"
#include "k_structure.h"

namespace condensa {

constexpr int kStructListLevels = 2;      // radix levels counted over all aggregates before the list takes over

struct StructListArgs {
    u64* count;            // entries offered (never more than cap: the list holds every structure)
    u64* key;              // [cap]
    u32* id;               // [cap] global structure ids
    u64 cap;
};

__global__ __launch_bounds__(kBlock) void k_struct_list_collect(StructArgs a, StructListArgs l) {
    __shared__ SlotStep s_e;
    __shared__ u64 s_wave[kBlock / 64];
    __shared__ u64 s_base;
    const int tid = threadIdx.x;
    if (tid < 64) {
        const SlotStep e = wave_enter_level(a.slots[0], kStructListLevels, 63, struct_hist(a, kStructListLevels - 1),
                                            struct_coarse(a, kStructListLevels - 1));
        if (tid == 0) s_e = e;
    }
    __syncthreads();
    if (s_e.state != kSelecting) return;                   // uniform: k == 0, nothing to rank
    const u64 prefix = s_e.prefix;
    const Level L = level_of(63, kStructListLevels - 1);   // entries agree with the prefix down to this level's digit
    for (u64 c = blockIdx.x; c < a.n_schunks; c += gridDim.x) {
        const int t = tensor_of_schunk(a.td, a.n_tensors, c);
        const TensorDesc& td = a.td[t];
        const u64 base = (c - td.pad) * kChunk;
        const u64 end = (base + kChunk < td.n_struct) ? base + kChunk : td.n_struct;
        const u64* __restrict__ kp = a.keys + td.struct_start;
        constexpr int kPer = kChunk / kBlock;              // 32 keys per thread and chunk, strided by the workgroup
        u64 key[kPer];
        u32 listed = 0;
#pragma unroll
        for (int u = 0; u < kPer; ++u) {
            const u64 i = base + tid + static_cast<u64>(u) * kBlock;
            key[u] = (i < end) ? kp[i] : ~prefix;          // a filler that fails the prefix test
        }
#pragma unroll
        for (int u = 0; u < kPer; ++u)
            if (base + tid + static_cast<u64>(u) * kBlock < end && ((key[u] ^ prefix) >> L.shift) == 0) listed |= 1u << u;
        u64 total;
        const u64 before = block_excl_scan_u64(static_cast<u64>(__popc(listed)), s_wave, &total);
        if (total != 0) {                                  // uniform over the workgroup
            if (tid == 0) s_base = atomicAdd(reinterpret_cast<unsigned long long*>(l.count), static_cast<unsigned long long>(total));
            __syncthreads();
            u64 pos = s_base + before;
#pragma unroll
            for (int u = 0; u < kPer; ++u) {
                if (listed & (1u << u)) {
                    if (pos < l.cap) {
                        l.key[pos] = key[u];
                        l.id[pos] = static_cast<u32>(td.struct_start + base + tid + static_cast<u64>(u) * kBlock);
                    }
                    ++pos;
                }
            }
            __syncthreads();                               // s_base is rewritten for the next chunk
        }
    }
}

__global__ __launch_bounds__(kSmallFinishThreads) void k_struct_list_finish(StructArgs a, StructListArgs l, condensa_select* results,
                                                                           int id_bits) {
    __shared__ SlotStep s_e;
    Slot& slot = a.slots[0];
    if (threadIdx.x < 64) {
        const SlotStep e = wave_enter_level(slot, kStructListLevels, 63, struct_hist(a, kStructListLevels - 1),
                                            struct_coarse(a, kStructListLevels - 1));
        if (threadIdx.x == 0) s_e = e;
    }
    __syncthreads();
    u64 n_list = *l.count;
    if (n_list > l.cap) n_list = l.cap;                    // (cannot happen: the list holds every structure)
    finish_on_list<u64, u32>(slot, s_e, l.key, l.id, n_list, 63, kStructListLevels, id_bits, results);
}

}  // namespace condensa
