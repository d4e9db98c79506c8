// Final step (Section 5.1 step 3 / Section 5.2 step 3): merge the split partial softmax states of each
// branch, normalise, and apply the per-branch gates; only the aggregated output is written, in the
// input dtype (round-to-nearest-even for bf16).
//   o_branch = sum_s 2^(m_s - M) acc_s / sum_s 2^(m_s - M) Z_s,   out = g_cmp o_cmp + g_slc o_slc + g_win o_win
//
// Three kernels.  k_combine_rows (few slices per row, many rows): a group of d_v/4 threads owns one output row (four
// columns per thread), eight or sixteen rows per workgroup, no cross-thread reduction: every thread of the group
// first folds the (m, Z) pairs of each branch's slices into the branch maximum and total (the loads of a group hit
// the same addresses), then accumulates gate * 2^(m - M) / Z_total * partial accumulator over the slices;
// k_combine_stream is its form for large calls (below).  k_combine_slices (many slices per row): one workgroup per
// output row; wavefronts 0..2 each take one branch with one lane per slice (wave-wide max and sum), then all 256
// threads accumulate weight * partial accumulator, 256 / (d_v/4) slices in parallel, and a small LDS reduction
// produces the row.
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
    int64_t out_s[3];     // bytes: sequence, query, head
    // k_combine_rows only: branches [br_lo, br_hi) in gate order (compressed, selected, window) are merged; with
    // use_gates == 0 their normalised sum is written as it is (one branch: that branch's output)
    int br_lo, br_hi, use_gates;
};

// byte offset of output row (b, i, h)
__device__ __forceinline__ int64_t out_row_offset(const CombineArgs& a, int64_t row) {
    const int h = (int)(row % a.H), i = (int)((row / a.H) % a.T);
    const int64_t b = row / ((int64_t)a.H * a.T);
    return b * a.out_s[0] + i * a.out_s[1] + h * a.out_s[2];
}

constexpr int kMaxSlotsPerBranch = 64;      // compressed scan; the other two branches: 32 each
constexpr int kMaxSlotsTotal = kMaxSlotsPerBranch + 32 + 32;

constexpr int kCombineRowsMaxSlots = 16;   // slices per row up to which a thread group owns a row (k_combine_rows)

// Every load is issued at once (one memory round trip: these calls are small and bound by latency).
template <bool BF16, int DV>
__global__ void __launch_bounds__(kThreads) k_combine_rows(const CombineArgs a) {
    constexpr int TPR = DV / 4;                 // threads across one row, 4 columns each
    constexpr int RPW = kThreads / TPR;         // rows per workgroup
    constexpr int MS = kCombineRowsMaxSlots;
    const int tid = threadIdx.x;
    const int64_t row = (int64_t)blockIdx.x * RPW + tid / TPR;
    if (row >= a.rows_total) return;
    const int c = tid % TPR;
    const int i = (int)((row / a.H) % a.T);
    const int b = (int)(row / ((int64_t)a.H * a.T));
    // slot ranges: cmp [0, n_cmp), win [n_cmp, n_cmp + n_win), slc after; gate order: cmp, slc, win
    const int lo3[3] = {0, a.n_cmp_chunks + a.n_win_splits, a.n_cmp_chunks};
    const int cnt3[3] = {a.n_cmp_chunks, a.n_slc_splits, a.n_win_splits};
    // the slots this launch reads: all of them, or one branch's (the host keeps either count within MS)
    const bool one_branch = a.br_hi - a.br_lo == 1;
    const int base = one_branch ? (a.br_lo == 0 ? lo3[0] : (a.br_lo == 1 ? lo3[1] : lo3[2])) : 0;
    const int n_read = one_branch ? (a.br_lo == 0 ? cnt3[0] : (a.br_lo == 1 ? cnt3[1] : cnt3[2]))
                                  : a.n_cmp_chunks + a.n_win_splits + a.n_slc_splits;

    // Everything this thread needs is fetched in one round of independent loads (slices that contributed nothing never
    // wrote their accumulator; whatever is read there is discarded by its zero weight).
    float2 st[MS];
    f32x4 v[MS];
#pragma unroll
    for (int s = 0; s < MS; ++s) {
        st[s] = make_float2(0.f, 0.f);
        v[s] = f32x4{0.f, 0.f, 0.f, 0.f};
        if (s < n_read) {              // uniform
            const int64_t pr = (int64_t)(base + s) * a.rows_total + row;
            st[s] = *reinterpret_cast<const float2*>(a.part_stats + pr * 2);
            v[s] = *reinterpret_cast<const f32x4*>(a.part_acc + pr * DV + c * 4);
        }
    }
    const float g3[3] = {a.gates[row * 3 + 0], a.gates[row * 3 + 1], a.gates[row * 3 + 2]};
    const int Tq = a.n_query ? min(max(a.n_query[b], 0), a.T) : a.T;

    f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
    if (i < Tq) {
#pragma unroll
        for (int br = 0; br < 3; ++br) {
            if (br < a.br_lo || br >= a.br_hi) continue;
            const int lo = lo3[br] - base, hi = lo + cnt3[br];      // in units of the slots read
            // branch maximum and total (slices that saw no key have Z = 0)
            float M = -INFINITY;
#pragma unroll
            for (int s = 0; s < MS; ++s)
                if (s >= lo && s < hi && s < n_read && st[s].y > 0.f) M = fmaxf(M, st[s].x);
            float Zt = 0.f;
#pragma unroll
            for (int s = 0; s < MS; ++s)
                if (s >= lo && s < hi && s < n_read && st[s].y > 0.f) Zt += st[s].y * fast_exp2(st[s].x - M);
            if (!(Zt > 0.f)) continue;
            const float scale = (a.use_gates ? g3[br] : 1.f) / Zt;
#pragma unroll
            for (int s = 0; s < MS; ++s)
                if (s >= lo && s < hi && s < n_read && st[s].y > 0.f) acc += (scale * fast_exp2(st[s].x - M)) * v[s];
        }
    }
    if constexpr (BF16) {
        __bf16 h[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) h[e] = (__bf16)acc[e];
        *reinterpret_cast<u32x2*>(reinterpret_cast<char*>(a.out) + out_row_offset(a, row) + c * 8) = *reinterpret_cast<u32x2*>(h);
    } else {
        *reinterpret_cast<f32x4*>(reinterpret_cast<char*>(a.out) + out_row_offset(a, row) + c * 16) = acc;
    }
}

// Large calls (partial states beyond the last-level cache): persistent workgroups over batches of rows.  Sixteen lanes
// per row turn the (m, Z) pairs of the row's slices into one weight per slice, gate * 2^(m - M_branch) / Z_branch, through
// lane exchanges; the weights go to LDS, and a group of d_v/4 threads per row then fetches only the accumulators with a
// non-zero weight (a short sequence of a mixed batch leaves most of its slices empty) and sums them in slot order.  The
// statistics of the next batch are fetched before the accumulators of the current one are summed, and become
// weights after it: one memory round trip per batch instead of two, and no start-up per batch.
template <bool BF16, int DV>
__global__ void __launch_bounds__(kThreads) k_combine_stream(const CombineArgs a) {
    constexpr int TPR = DV / 4;                 // threads across one row, 4 columns each
    constexpr int RPW = kThreads / TPR;         // rows per batch
    constexpr int MS = kCombineRowsMaxSlots;
    static_assert(RPW * MS <= kThreads && MS == 16, "one lane per (row, slice) of a batch; 16-lane exchanges");
    __shared__ float s_w[2][RPW][MS];
    const int tid = threadIdx.x;
    const int n_read = a.n_cmp_chunks + a.n_win_splits + a.n_slc_splits;
    const int64_t n_batches = (a.rows_total + RPW - 1) / RPW;
    // weight lanes: row wr of the batch, slice ws; its branch in gate order (compressed, selected, window)
    const int wr = tid / MS, ws = tid % MS;
    const bool wlane = tid < RPW * MS && ws < n_read;
    const int wbr = ws < a.n_cmp_chunks ? 0 : (ws < a.n_cmp_chunks + a.n_win_splits ? 2 : 1);
    struct Fetched { float2 st; float gate; bool live; };
    auto fetch = [&](int64_t batch) {
        Fetched f{make_float2(0.f, 0.f), 0.f, false};
        const int64_t row = batch * RPW + wr;
        if (wlane && batch < n_batches && row < a.rows_total) {
            const int i = (int)((row / a.H) % a.T);
            const int b = (int)(row / ((int64_t)a.H * a.T));
            const int Tq = a.n_query ? min(max(a.n_query[b], 0), a.T) : a.T;
            f.st = *reinterpret_cast<const float2*>(a.part_stats + ((int64_t)ws * a.rows_total + row) * 2);
            f.gate = a.gates[row * 3 + wbr];
            f.live = i < Tq;
        }
        return f;
    };
    auto weight = [&](const Fetched& f) {       // (all 64 lanes of a wavefront take part in the exchanges)
        const bool valid = f.live && f.st.y > 0.f;
        float w = 0.f;
#pragma unroll
        for (int br = 0; br < 3; ++br) {
            const bool mine = valid && wbr == br;
            float M = mine ? f.st.x : -INFINITY;
#pragma unroll
            for (int off = 8; off >= 1; off >>= 1) M = fmaxf(M, __shfl_xor(M, off));
            const float e = mine ? fast_exp2(f.st.x - M) : 0.f;
            float Zt = e * f.st.y;
#pragma unroll
            for (int off = 8; off >= 1; off >>= 1) Zt += __shfl_xor(Zt, off);
            if (mine) w = f.gate * e / Zt;
        }
        return w;
    };

    int64_t batch = blockIdx.x;
    if (batch >= n_batches) return;
    if (tid < RPW * MS) s_w[0][wr][ws] = weight(fetch(batch));
    __syncthreads();
    const int r = tid / TPR, c = tid % TPR;
    for (int buf = 0; batch < n_batches; batch += gridDim.x, buf ^= 1) {
        const Fetched nxt = fetch(batch + gridDim.x);
        __builtin_amdgcn_sched_barrier(0);      // the statistics of the next batch are on their way before anything below
        const int64_t row = batch * RPW + r;
        if (row < a.rows_total) {
            // eight slices at a time: their loads in flight together (registers for all sixteen would cost a wavefront
            // per SIMD)
            f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
            const float* src = a.part_acc + row * DV + c * 4;
            const int64_t slot_stride = a.rows_total * DV;
#pragma unroll
            for (int h = 0; h < MS; h += 8) {
                if (h >= n_read) break;
                float w[8];
                f32x4 v[8];
#pragma unroll
                for (int s = 0; s < 8; ++s) {
                    w[s] = h + s < n_read ? s_w[buf][r][h + s] : 0.f;
                    v[s] = f32x4{0.f, 0.f, 0.f, 0.f};
                    if (w[s] != 0.f) v[s] = *reinterpret_cast<const f32x4*>(src + (h + s) * slot_stride);
                }
#pragma unroll
                for (int s = 0; s < 8; ++s)
                    if (w[s] != 0.f) acc += w[s] * v[s];
                __builtin_amdgcn_sched_barrier(0);
            }
            if constexpr (BF16) {
                __bf16 h[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) h[e] = (__bf16)acc[e];
                *reinterpret_cast<u32x2*>(reinterpret_cast<char*>(a.out) + out_row_offset(a, row) + c * 8) = *reinterpret_cast<u32x2*>(h);
            } else {
                *reinterpret_cast<f32x4*>(reinterpret_cast<char*>(a.out) + out_row_offset(a, row) + c * 16) = acc;
            }
        }
        if (tid < RPW * MS) s_w[buf ^ 1][wr][ws] = weight(nxt);
        __syncthreads();
    }
}

__device__ __forceinline__ float wave_max_f32(float v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v = fmaxf(v, __shfl_xor(v, off));
    return v;
}
__device__ __forceinline__ float wave_sum_f32(float v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
    return v;
}

template <bool BF16, int DV>
__global__ void __launch_bounds__(kThreads) k_combine_slices(const CombineArgs a) {
    constexpr int TPR = DV / 4;                 // threads across one row, 4 columns each
    constexpr int SL = kThreads / TPR;          // slices accumulated in parallel
    __shared__ float s_w[kMaxSlotsTotal];
    __shared__ f32x4 s_red[SL][TPR];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t row = blockIdx.x;
    const int i = (int)((row / a.H) % a.T);
    const int b = (int)(row / ((int64_t)a.H * a.T));
    const int Tq = a.n_query ? min(max(a.n_query[b], 0), a.T) : a.T;
    const int n_slots = a.n_cmp_chunks + a.n_win_splits + a.n_slc_splits;
    const int c = tid % TPR, sl = tid / TPR;

    f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
    if (i < Tq) {     // uniform per workgroup
        if (wave < 3) {
            // slot ranges: cmp [0, n_cmp), win [n_cmp, n_cmp + n_win), slc after; gate order: cmp, slc, win
            const int lo = wave == 0 ? 0 : (wave == 1 ? a.n_cmp_chunks + a.n_win_splits : a.n_cmp_chunks);
            const int cnt = wave == 0 ? a.n_cmp_chunks : (wave == 1 ? a.n_slc_splits : a.n_win_splits);
            float m = -INFINITY, z = 0.f;
            if (lane < cnt) {
                const float2 st = *reinterpret_cast<const float2*>(a.part_stats + ((int64_t)(lo + lane) * a.rows_total + row) * 2);
                if (st.y > 0.f) { m = st.x; z = st.y; }
            }
            const float M = wave_max_f32(m);
            const float e = z > 0.f ? fast_exp2(m - M) : 0.f;
            const float Zt = wave_sum_f32(e * z);
            const float gate = a.gates[row * 3 + wave];
            if (lane < cnt) s_w[lo + lane] = Zt > 0.f ? gate * e / Zt : 0.f;
        }
        __syncthreads();
        for (int s0 = sl; s0 < n_slots; s0 += 4 * SL) {
            float w[4];
            f32x4 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int s = s0 + u * SL;
                w[u] = s < n_slots ? s_w[s] : 0.f;
                // slices that contributed nothing never wrote their accumulator: read slice 0's memory instead
                // (always mapped) and discard it, so that the load stays unconditional
                const int64_t pr = (int64_t)(w[u] != 0.f ? s : 0) * a.rows_total + row;
                v[u] = *reinterpret_cast<const f32x4*>(a.part_acc + pr * DV + c * 4);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (w[u] != 0.f) acc += w[u] * v[u];
        }
    }
    s_red[sl][c] = acc;
    __syncthreads();
    if (sl == 0) {
        f32x4 o = s_red[0][c];
#pragma unroll
        for (int k = 1; k < SL; ++k) o += s_red[k][c];
        if constexpr (BF16) {
            __bf16 h[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) h[e] = (__bf16)o[e];
            *reinterpret_cast<u32x2*>(reinterpret_cast<char*>(a.out) + out_row_offset(a, row) + c * 8) = *reinterpret_cast<u32x2*>(h);
        } else {
            *reinterpret_cast<f32x4*>(reinterpret_cast<char*>(a.out) + out_row_offset(a, row) + c * 16) = o;
        }
    }
}

// Gate kernel of the unfused execution (the structure the fused path replaces, Section 5): the three branch
// outputs were written to scratch in the storage type, [rows, d_v] each; this launch reads them back and writes
// out = g_cmp o_cmp + g_slc o_slc + g_win o_win.  One thread per four output columns.
struct GateArgs {
    const void *o_cmp, *o_slc, *o_win;
    const float* gates;
    const int32_t* n_query;
    void* out;
    int T, H;
    int64_t rows_total;
    int64_t out_s[3];
};

template <bool BF16, int DV>
__global__ void __launch_bounds__(kThreads) k_gate(const GateArgs a) {
    constexpr int TPR = DV / 4, RPW = kThreads / TPR;
    const int tid = threadIdx.x;
    const int64_t row = (int64_t)blockIdx.x * RPW + tid / TPR;
    if (row >= a.rows_total) return;
    const int c = tid % TPR;
    const int h = (int)(row % a.H), i = (int)((row / a.H) % a.T);
    const int64_t b = row / ((int64_t)a.H * a.T);
    const int Tq = a.n_query ? min(max(a.n_query[b], 0), a.T) : a.T;
    f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
    if (i < Tq) {
        const void* src[3] = {a.o_cmp, a.o_slc, a.o_win};
#pragma unroll
        for (int br = 0; br < 3; ++br) {
            const float gate = a.gates[row * 3 + br];
            f32x4 v;
            if constexpr (BF16) {
                const u32x2 raw = *reinterpret_cast<const u32x2*>(reinterpret_cast<const char*>(src[br]) + (row * DV + c * 4) * 2);
                v = f32x4{__uint_as_float(raw[0] << 16), __uint_as_float(raw[0] & 0xFFFF0000u),
                          __uint_as_float(raw[1] << 16), __uint_as_float(raw[1] & 0xFFFF0000u)};
            } else {
                v = *reinterpret_cast<const f32x4*>(reinterpret_cast<const char*>(src[br]) + (row * DV + c * 4) * 4);
            }
            acc += gate * v;
        }
    }
    char* dst = reinterpret_cast<char*>(a.out) + b * a.out_s[0] + i * a.out_s[1] + h * a.out_s[2];
    if constexpr (BF16) {
        __bf16 hh[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) hh[e] = (__bf16)acc[e];
        *reinterpret_cast<u32x2*>(dst + c * 8) = *reinterpret_cast<u32x2*>(hh);
    } else {
        *reinterpret_cast<f32x4*>(dst + c * 16) = acc;
    }
}

}  // namespace ssv
