// Work tables for batches of mixed lengths: which (sequence, slice) a workgroup of a pass over k_cmp takes, so that one
// round of resident workgroups holds slices of about equal length whatever the lengths are.  The lengths live in device
// memory, so the table is built on the device: by one workgroup of the launch before (the balanced matrix-core scan
// builds the importance pass's table, k_scan32.hpp) or by the one-workgroup kernel below (ahead of the streaming
// kernel's compressed scan, k_stream.hpp).
//
//   Sequence b with n_b tiles of 64 compressed rows gets k_b = ceil(n_b D / W) slices, W = sum_b n_b and
//   D = items_max - (sequences with work): slices of at most W / D tiles, and sum_b k_b <= items_max (integer
//   arithmetic: the bound is exact).  A sequence counts at least one tile if it has queries (its rows need their
//   statistics written) and nothing if it has none.
//
//   Layout (int32): [0] = number of items, [4 + 4 i ..] = (sequence, slice, slices of that sequence, 0) of item i, items
//   in sequence order.
#pragma once
#include "device_common.hpp"

namespace ssv {

constexpr int kWorkTableHeader = 4;
__host__ __device__ inline size_t work_table_bytes(int items_max) { return (size_t)(kWorkTableHeader + 4 * items_max) * sizeof(int32_t); }

// tiles of sequence b as the tables count them
__device__ __forceinline__ int work_tiles_of(int b, int B, int T, const int32_t* n_query, const int32_t* n_cmp, int max_n_cmp) {
    if (b >= B) return 0;
    const int tq = n_query ? min(max(n_query[b], 0), T) : T;
    return tq > 0 ? max(1, (min(max(n_cmp[b], 0), max_n_cmp) + kTile - 1) / kTile) : 0;
}

// Built by all THREADS threads of a workgroup; thread t brings the tiles of sequences PT t .. PT t + PT - 1 (0 beyond the
// batch).  slices_cap bounds the slices of one sequence (the partial-state slots a pass has per row; large if none).
// s_wsum: THREADS / 64 ints of LDS.
template <int THREADS, int PT>
__device__ __forceinline__ void block_build_work_table(const int (&tiles)[PT], int items_max, int slices_cap, int32_t* table, int* s_wsum, int tid) {
    const int lane = tid & 63, wave = tid >> 6;
    auto block_sum = [&](int v) {
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
        __syncthreads();        // s_wsum is free
        if (lane == 0) s_wsum[wave] = v;
        __syncthreads();
        int t = 0;
        for (int w = 0; w < THREADS / 64; ++w) t += s_wsum[w];
        return t;
    };
    int mine = 0, act = 0;
#pragma unroll
    for (int i = 0; i < PT; ++i) {
        mine += tiles[i];
        act += tiles[i] > 0;
    }
    const int W = block_sum(mine), active = block_sum(act);
    const int D = max(1, items_max - active);
    int k[PT], ksum = 0;
#pragma unroll
    for (int i = 0; i < PT; ++i) {
        k[i] = tiles[i] > 0 ? min((int)(((int64_t)tiles[i] * D + W - 1) / W), min(slices_cap, items_max)) : 0;
        ksum += k[i];
    }
    int inc = ksum;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int up = __shfl_up(inc, off);
        if (lane >= off) inc += up;
    }
    __syncthreads();
    if (lane == 63) s_wsum[wave] = inc;
    __syncthreads();
    int item = inc - ksum, total = 0;
    for (int w = 0; w < THREADS / 64; ++w) {
        if (w < wave) item += s_wsum[w];
        total += s_wsum[w];
    }
    // (the total stays within items_max whenever the batch has fewer sequences with work than items_max: the host asks for
    // twice as many; the bound below only guards the table)
#pragma unroll
    for (int i = 0; i < PT; ++i)
        for (int part = 0; part < k[i]; ++part, ++item)
            if (item < items_max) reinterpret_cast<int4*>(table + kWorkTableHeader)[item] = make_int4(PT * tid + i, part, k[i], 0);
    if (tid == 0) table[0] = min(total, items_max);
}

// item -> (sequence, slice, slices); false: the table has fewer items
__device__ __forceinline__ bool work_table_item(const int32_t* table, int item, int B, int& b, int& part, int& parts) {
    if (item >= table[0]) return false;
    const int4 e = reinterpret_cast<const int4*>(table + kWorkTableHeader)[item];
    b = min(max(e.x, 0), B - 1);
    part = e.y;
    parts = e.z;
    return true;
}

constexpr int kWorkTableMaxB = 4 * kThreads;       // sequences per batch the kernel below takes

struct WorkTableArgs {
    const int32_t *n_cmp, *n_query;
    int B, T, max_n_cmp;
    int32_t* scan_table;     // the compressed scan's table, or null
    int scan_items_max, scan_slices_cap;
    int32_t* imp_table;      // the importance pass's table, or null
    int imp_items_max;
};

// One workgroup; B <= kWorkTableMaxB.
__global__ void __launch_bounds__(kThreads) k_work_table(const WorkTableArgs a) {
    __shared__ int s_wsum[kThreads / 64];
    const int tid = threadIdx.x;
    int tiles[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) tiles[i] = work_tiles_of(4 * tid + i, a.B, a.T, a.n_query, a.n_cmp, a.max_n_cmp);
    if (a.scan_table) block_build_work_table<kThreads, 4>(tiles, a.scan_items_max, a.scan_slices_cap, a.scan_table, s_wsum, tid);
    if (a.imp_table) block_build_work_table<kThreads, 4>(tiles, a.imp_items_max, 1 << 30, a.imp_table, s_wsum, tid);
}

}  // namespace ssv
