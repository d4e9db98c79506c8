// Compressed-cache construction: the step just before the verification path.  The compression branch
// aggregates committed tokens into blocks of length l every d tokens (Section 2.2); here the aggregate is the
// mean of the block's rows.  Only blocks made of committed tokens are produced, so draft tokens enter the
// compressed cache when they are accepted, not before.
//
// One workgroup = one (sequence, KV head, K or V) x a run of consecutive new compressed rows.  Every raw row
// is read once: the run's raw rows are summed per stride-d chunk into LDS (fp32, slot order), then each
// compressed row is the sum of its l/d consecutive chunks times 1/l, rounded once to the storage type.
#pragma once
#include "device_common.hpp"

namespace ssv {

struct CompressArgs {
    const char *k, *v;
    char *kc, *vc;
    const int32_t *before, *after;   // committed tokens per sequence before / after this update (before may be null = 0)
    int32_t* n_cmp;                  // out: complete compressed rows per sequence after the update
    int B, H_kv;
    int l, d, ratio;                 // ratio = l / d chunks per compressed row
    int rows_per_wg, cap;            // compressed rows per workgroup; row capacity of kc / vc
    int kv_cap, max_new;             // row capacity of k / v; most rows one sequence may gain in this launch
    int k_groups, v_groups;          // 16-byte column groups per K / V row
    float inv_l;
    int64_t k_s[3], v_s[3], kc_s[3], vc_s[3];   // bytes: sequence, KV head, row
};

__device__ __forceinline__ int complete_cmp_rows(int L, int l, int d) { return L < l ? 0 : (L - l) / d + 1; }

template <bool BF16>
__global__ void __launch_bounds__(kThreads) k_compress(const CompressArgs a) {
    constexpr int EPG = BF16 ? 8 : 4;           // elements per 16-byte group
    extern __shared__ __align__(16) char smem[];
    float* s_chunk = reinterpret_cast<float*>(smem);   // [rows_per_wg + ratio - 1][groups * EPG] chunk sums

    const int tid = threadIdx.x;
    const int b = blockIdx.y / a.H_kv, h = blockIdx.y % a.H_kv;
    const bool is_v = blockIdx.z != 0;
    const int L_before = a.before ? max(a.before[b], 0) : 0;
    const int L_after = min(max(a.after[b], 0), a.kv_cap);
    const int c_lo = min(complete_cmp_rows(L_before, a.l, a.d), a.cap);
    const int c_hi = min(min(complete_cmp_rows(L_after, a.l, a.d), a.cap), c_lo + a.max_new);
    if (blockIdx.x == 0 && h == 0 && !is_v && tid == 0) a.n_cmp[b] = c_hi;
    const int r0 = c_lo + blockIdx.x * a.rows_per_wg;
    const int r1 = min(r0 + a.rows_per_wg, c_hi);
    if (r0 >= r1) return;

    const int groups = is_v ? a.v_groups : a.k_groups;
    const int width = groups * EPG;
    const int64_t src_row = is_v ? a.v_s[2] : a.k_s[2];
    const char* src = is_v ? a.v + b * a.v_s[0] + h * a.v_s[1] : a.k + b * a.k_s[0] + h * a.k_s[1];
    const int n_rows = r1 - r0, n_chunks = n_rows + a.ratio - 1;

    // chunk sums: chunk x of the run covers slots [(r0 + x) d, (r0 + x + 1) d), all below L_after
    for (int task = tid; task < n_chunks * groups; task += kThreads) {
        const int x = task / groups, cg = task - x * groups;
        const char* p = src + (int64_t)(r0 + x) * a.d * src_row + cg * 16;
        float acc[EPG];
#pragma unroll
        for (int e = 0; e < EPG; ++e) acc[e] = 0.f;
        auto add_row = [&](const u32x4 raw) {
            if (BF16) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    acc[2 * e] += __uint_as_float(raw[e] << 16);
                    acc[2 * e + 1] += __uint_as_float(raw[e] & 0xFFFF0000u);
                }
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) acc[e] += __uint_as_float(raw[e]);
            }
        };
        if (a.d == 16) {        // the standard stride: all sixteen row loads in flight before the first add
            u32x4 raw[16];
#pragma unroll
            for (int r = 0; r < 16; ++r) raw[r] = *reinterpret_cast<const u32x4*>(p + r * src_row);
#pragma unroll
            for (int r = 0; r < 16; ++r) add_row(raw[r]);
        } else {
#pragma unroll 4
            for (int r = 0; r < a.d; ++r) add_row(*reinterpret_cast<const u32x4*>(p + r * src_row));
        }
#pragma unroll
        for (int e = 0; e < EPG; e += 4)
            *reinterpret_cast<f32x4*>(s_chunk + x * width + cg * EPG + e) = f32x4{acc[e], acc[e + 1], acc[e + 2], acc[e + 3]};
    }
    __syncthreads();

    const int64_t dst_row = is_v ? a.vc_s[2] : a.kc_s[2];
    char* dst = is_v ? a.vc + b * a.vc_s[0] + h * a.vc_s[1] : a.kc + b * a.kc_s[0] + h * a.kc_s[1];
    for (int task = tid; task < n_rows * groups; task += kThreads) {
        const int c = task / groups, cg = task - c * groups;
        float acc[EPG];
#pragma unroll
        for (int e = 0; e < EPG; ++e) acc[e] = 0.f;
        for (int m = 0; m < a.ratio; ++m) {
#pragma unroll
            for (int e = 0; e < EPG; ++e) acc[e] += s_chunk[(c + m) * width + cg * EPG + e];
        }
        u32x4 packed;
        if (BF16) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const __bf16 lo = (__bf16)(acc[2 * e] * a.inv_l), hi = (__bf16)(acc[2 * e + 1] * a.inv_l);
                packed[e] = (uint32_t)__builtin_bit_cast(uint16_t, lo) | ((uint32_t)__builtin_bit_cast(uint16_t, hi) << 16);
            }
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) packed[e] = __float_as_uint(acc[e] * a.inv_l);
        }
        *reinterpret_cast<u32x4*>(dst + (int64_t)(r0 + c) * dst_row + cg * 16) = packed;
    }
}

}  // namespace ssv
