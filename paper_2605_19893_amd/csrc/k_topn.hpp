// Routing, part 3: block importance and top-n selection per (sequence, verifier query, KV group)
// ("Top-n reduction", Section 5.1; mandatory initial and local blocks that count toward n, Section 7.3).
//
//   imp[j] = sum_{m < l'/d} sum_{n' < l/d} colsum[(l'/d) j + m - n']      (terms outside [0, visible) are 0)
//   candidates j = 0..J, J = block of the query's own slot; forced blocks are ranked first;
//   the n_eff = min(n, J+1) best by (importance descending, index ascending) are written ascending.
//
// One workgroup per (b, i, g).  Keys are packed as (float bits << 32) | ~index so that a plain
// unsigned 64-bit maximum implements "larger importance, then smaller index"; importances are sums
// of probabilities, hence non-negative, and their IEEE bit patterns order like the values.
#pragma once
#include "device_common.hpp"

namespace ssv {

struct TopnArgs {
    const float* colsum;     // [B, T, H_kv, nc_pitch]
    const int32_t *seq_lens, *n_cmp, *n_query, *parents;
    int32_t* sel_idx;        // [B, T, H_kv, n_sel]
    int B, T, H_kv;
    int l, d, l_sel, n_sel, n_init, n_local;
    int nc_pitch;
    int max_blocks;          // capacity of the key array in LDS
};

constexpr int kMaxNSel = 32;

// 64-bit maximum over a wavefront: four DPP butterfly steps inside each row of 16 lanes
// (quad swaps, then half-row and row mirrors, which pair groups that already agree), then the four
// row results are read out as scalars.  The result is wave-uniform.
template <int CTRL>
__device__ __forceinline__ uint64_t dpp_max_step(uint64_t v) {
    const uint32_t lo = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)v, CTRL, 0xF, 0xF, false);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)(v >> 32), CTRL, 0xF, 0xF, false);
    const uint64_t o = ((uint64_t)hi << 32) | lo;
    return o > v ? o : v;
}

__device__ __forceinline__ uint64_t wave_max_u64(uint64_t v) {
    v = dpp_max_step<0xB1>(v);    // quad_perm [1,0,3,2]
    v = dpp_max_step<0x4E>(v);    // quad_perm [2,3,0,1]
    v = dpp_max_step<0x141>(v);   // row_half_mirror
    v = dpp_max_step<0x140>(v);   // row_mirror
    uint64_t best = 0;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)v, 16 * r);
        const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(v >> 32), 16 * r);
        const uint64_t o = ((uint64_t)hi << 32) | lo;
        best = o > best ? o : best;
    }
    return best;
}

constexpr int kMaxImpTerms = 8;   // (l'/d) + (l/d) - 1 compressed columns feed one selection block

__global__ void __launch_bounds__(kThreads) k_topn(const TopnArgs a) {
    extern __shared__ __align__(16) char smem[];
    uint64_t* s_key = reinterpret_cast<uint64_t*>(smem);                  // [max_blocks]
    uint64_t* s_red = s_key + a.max_blocks;                               // [2][4]
    int* s_pick = reinterpret_cast<int*>(s_red + 8);                      // [kMaxNSel]
    uint64_t* s_anc = reinterpret_cast<uint64_t*>(s_pick + kMaxNSel);
    int* s_par = reinterpret_cast<int*>(s_anc + kMaxT);
    int* s_depth = s_par + kMaxT;
    int* s_cmax = s_depth + kMaxT;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = blockIdx.x % a.H_kv;
    const int i = (blockIdx.x / a.H_kv) % a.T;
    const int b = blockIdx.x / (a.H_kv * a.T);
    int32_t* out = a.sel_idx + (((int64_t)b * a.T + i) * a.H_kv + g) * a.n_sel;

    const SeqMeta sm = build_tree_meta(tid, b, a.T, a.seq_lens, a.n_query, a.n_cmp, a.parents, a.l, a.d, s_par, s_depth, s_cmax,
                                       s_anc);
    if (i >= sm.Tq) {
        if (tid < a.n_sel) out[tid] = -1;
        return;
    }
    const int ncv = min(s_cmax[i], a.nc_pitch);
    const int J = min((sm.L + i) / a.l_sel, a.max_blocks - 1);
    const int a_ratio = a.l_sel / a.d, b_ratio = a.l / a.d;
    const float* cs = a.colsum + (((int64_t)b * a.T + i) * a.H_kv + g) * a.nc_pitch;

    // imp[j] = sum_delta wt[delta] * colsum[a_ratio * j + delta], delta in [-(b_ratio-1), a_ratio-1], where
    // wt counts the (m, n') pairs with m - n' = delta.  All loads of a block are unconditional (clamped
    // column, zero weight) so that they are in flight together.
    const int n_terms = a_ratio + b_ratio - 1;
    uint64_t best = 0;   // best key among the blocks owned by this thread (index % 256 == tid)
    for (int j = tid; j <= J; j += kThreads) {
        float imp = 0.f;
        if (n_terms <= kMaxImpTerms) {
            float x[kMaxImpTerms], wt[kMaxImpTerms];
#pragma unroll
            for (int u = 0; u < kMaxImpTerms; ++u) {
                const int delta = u - (b_ratio - 1);
                const int c = a_ratio * j + delta;
                const bool ok = u < n_terms && c >= 0 && c < ncv;
                const int pairs = min(min(a_ratio, b_ratio), min(delta + b_ratio, a_ratio - delta));
                wt[u] = ok ? (float)pairs : 0.f;
                x[u] = cs[ok ? c : 0];
            }
#pragma unroll
            for (int u = 0; u < kMaxImpTerms; ++u) imp += wt[u] != 0.f ? wt[u] * x[u] : 0.f;
        } else {
            for (int m = 0; m < a_ratio; ++m)
                for (int n2 = 0; n2 < b_ratio; ++n2) {
                    const int c = a_ratio * j + m - n2;
                    if (c >= 0 && c < ncv) imp += cs[c];
                }
        }
        const bool forced = j < a.n_init || j > J - a.n_local;
        const uint32_t bits = forced ? 0x7F800000u : __float_as_uint(imp);
        const uint64_t key = ((uint64_t)bits << 32) | (uint32_t)(0xFFFFFFFFu - (uint32_t)j);
        s_key[j] = key;
        best = key > best ? key : best;
    }
    const int n_eff = min(a.n_sel, J + 1);
    __syncthreads();

    for (int round = 0; round < n_eff; ++round) {
        const uint64_t wbest = wave_max_u64(best);
        uint64_t* red = s_red + (round & 1) * 4;
        if (lane == 0) red[wave] = wbest;
        __syncthreads();
        uint64_t top = red[0];
#pragma unroll
        for (int k = 1; k < 4; ++k) top = red[k] > top ? red[k] : top;
        const int j_top = (int)(0xFFFFFFFFu - (uint32_t)top);
        if (tid == 0) s_pick[round] = j_top;
        if ((j_top % kThreads) == tid) {       // the owner retires the winner and rescans its blocks
            s_key[j_top] = 0;
            best = 0;
            for (int j = tid; j <= J; j += kThreads) best = s_key[j] > best ? s_key[j] : best;
        }
    }
    __syncthreads();
    if (tid < a.n_sel) {
        int val = -1;
        if (tid < n_eff) {      // ascending order by rank counting (picks are distinct)
            // find the element whose rank equals tid
            for (int e = 0; e < n_eff; ++e) {
                const int x = s_pick[e];
                int rank = 0;
                for (int f = 0; f < n_eff; ++f) rank += s_pick[f] < x;
                if (rank == tid) val = x;
            }
        }
        out[tid] = val;
    }
}

}  // namespace ssv
