// Final step (Section 5.1 step 3 / Section 5.2 step 3): merge the split partial softmax states of each
// branch, normalise, and apply the per-branch gates; only the aggregated output is written, in the
// input dtype (round-to-nearest-even for bf16).
//   o_branch = sum_s 2^(m_s - M) acc_s / sum_s 2^(m_s - M) Z_s,   out = g_cmp o_cmp + g_slc o_slc + g_win o_win
#pragma once
#include "device_common.hpp"

namespace ssv {

struct CombineArgs {
    const float *part_stats, *part_acc, *gates;
    const int32_t* n_query;
    void* out;
    int T, H;
    int n_cmp_chunks, n_win_splits, n_slc_splits;
    int64_t rows_total;
};

template <bool BF16, int DV>
__global__ void __launch_bounds__(kThreads) k_combine(const CombineArgs a) {
    constexpr int TPR = DV / 4;                 // threads per output row, 4 columns each
    constexpr int RPB = kThreads / TPR;         // rows per workgroup
    const int tid = threadIdx.x;
    const int64_t row = (int64_t)blockIdx.x * RPB + tid / TPR;
    const int c4 = (tid % TPR) * 4;
    if (row >= a.rows_total) return;
    const int i = (int)((row / a.H) % a.T);
    const int b = (int)(row / ((int64_t)a.H * a.T));
    const int Tq = a.n_query ? min(max(a.n_query[b], 0), a.T) : a.T;

    f32x4 o = f32x4{0.f, 0.f, 0.f, 0.f};
    if (i < Tq) {
        const int lo[3] = {0, a.n_cmp_chunks + a.n_win_splits, a.n_cmp_chunks};
        const int cnt[3] = {a.n_cmp_chunks, a.n_slc_splits, a.n_win_splits};   // gate order: cmp, slc, win
#pragma unroll
        for (int br = 0; br < 3; ++br) {
            float M = -INFINITY;
            for (int s = 0; s < cnt[br]; ++s) {
                const float* ps = a.part_stats + ((int64_t)(lo[br] + s) * a.rows_total + row) * 2;
                if (ps[1] > 0.f) M = fmaxf(M, ps[0]);
            }
            if (M == -INFINITY) continue;          // empty branch contributes zero
            float Z = 0.f;
            f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
            for (int s = 0; s < cnt[br]; ++s) {
                const int64_t pr = (int64_t)(lo[br] + s) * a.rows_total + row;
                const float* ps = a.part_stats + pr * 2;
                if (ps[1] > 0.f) {
                    const float wgt = fast_exp2(ps[0] - M);
                    Z += wgt * ps[1];
                    const f32x4 v = *reinterpret_cast<const f32x4*>(a.part_acc + pr * DV + c4);
                    acc += wgt * v;
                }
            }
            const float gate = a.gates[row * 3 + br];
            o += (gate / Z) * acc;
        }
    }
    if constexpr (BF16) {
        __bf16 h[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) h[e] = (__bf16)o[e];
        *reinterpret_cast<u32x2*>(reinterpret_cast<char*>(a.out) + (row * DV + c4) * 2) = *reinterpret_cast<u32x2*>(h);
    } else {
        *reinterpret_cast<f32x4*>(reinterpret_cast<char*>(a.out) + (row * DV + c4) * 4) = o;
    }
}

}  // namespace ssv
