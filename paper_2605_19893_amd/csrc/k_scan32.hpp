// Compressed scan for many rows per KV head (Section 2.2, compression branch; Section 4.1: the heads of a GQA
// group times the verifier queries of a group form the rows of the matrix tiles).  With several hundred rows per
// (sequence, KV head) the scan of k_cmp / v_cmp is a dense attention pass bound by the matrix cores, not by HBM, so
// this kernel is laid out for them: bf16 on the 32x32x16 matrix instruction, one workgroup of eight wavefronts per
// CU (two per SIMD), 256 rows per workgroup, one block of 32 rows per wavefront.
//
//   S^T = K Q^T in 32-key x 32-row blocks (K rows as the M dimension): a lane holds 16 keys of one row, so row
//   maxima and sums stay in the lane except for one exchange between the lane halves, and P^T (bf16) is directly
//   the B operand of O^T = V^T P^T.
//
//   K and V tiles of 64 compressed rows go from global memory straight into a ring of three LDS stages, with bank
//   swizzles chosen through the per-lane global addresses, two tiles ahead of the one in use; one barrier per tile.
//   Every tile reaches LDS once per 256 rows.  The two wavefronts of a SIMD overlap each other's matrix and vector
//   phases (products, softmax arithmetic, P.V).
//
//   The running maximum is a reference that is only raised when a tile's maximum exceeds it by more than 2^8
//   (probabilities stay below 256: exact in the partial state's own terms, which carries the reference), so the
//   accumulators are rescaled rarely.  Only the last one or two tiles of a sequence need per-row visibility masks.
//
// Work split.  Even: workgroup = (sequence, KV head, slice, query group), every group's tiles cut into n_chunks even
// slices (equal-length sequences).  Balanced: the tiles of all (sequence, KV head) pairs laid end to end and cut into
// equal ranges, one range per workgroup (times the query groups, which walk the same range side by side); a range
// that crosses into the next pair or sequence finishes one state and starts another.  A batch of mixed lengths then
// takes one round of equally long workgroups whatever the lengths are, read from device memory by every workgroup
// (a prefix sum over the batch); the host only bounds the slices per pair by the slot count.
//
// Output: one partial softmax state per row and slice, in the format of the streaming kernel (k_stream.hpp).
#pragma once
#include "k_stream.hpp"
#include "work_table.hpp"

namespace ssv {

struct Scan32Args {
    const char *q, *kc, *vc;
    const int32_t *seq_lens, *n_cmp, *n_query, *parents;
    float *part_stats, *part_acc;
    int B, T, H, H_kv, H_g;
    int C, n_qg;                  // verifier queries per workgroup (C * H_g <= 256); such groups per sequence
    int l, d;
    int max_seq_len, max_n_cmp;   // host-side bounds the lengths read from device memory are clamped to
    float scale_log2;
    int n_chunks;                 // slices of the compressed rows of one group = partial-state slots [0, n_chunks)
    int min_tiles;
    int n_wg;                     // real workgroups (the grid is padded to a multiple of 8)
    int n_ranges, range_min;      // balanced: ranges (n_wg = n_ranges * n_qg); shortest range that keeps every
                                  // (sequence, KV head) pair within n_chunks slices
    int pair_cost;                // balanced: what a segment costs besides its tiles, in tiles
    int32_t* imp_table;           // balanced, refresh calls: work table of the importance pass (work_table.hpp), or null
    int imp_items_max;            // its capacity in items (at least twice the batch size)
    int64_t rows_total;
    int64_t kc_s[3], vc_s[3];     // strides in bytes: sequence, KV head, row
    int64_t q_s[3];               // strides in bytes: sequence, query, head
};

constexpr int kScan32Threads = 512;      // eight wavefronts of 32 rows
constexpr int kScan32MaxBalancedB = 2 * kScan32Threads;   // sequences per batch the balanced split can take (LDS prefix array)

template <int DK, int DV>
struct Scan32Cfg {
    static constexpr int KROW = DK * 2, VROW = DV * 2;      // bytes per row
    static constexpr int STEPS = DK / 16;                   // 16-element contraction steps of S^T = K Q^T
    static constexpr int MB = DV / 32;                      // 32-column blocks of O^T
    static constexpr int KT = kTile * KROW, VT = kTile * VROW;
    static constexpr int STAGE = KT + VT;                   // one stage of the ring: K(t), then V(t)
    static constexpr int DEPTH = 3;
    static constexpr int LDS = DEPTH * STAGE;               // dynamic LDS bytes
    static constexpr int ROWS = 256;                        // rows per workgroup
    static constexpr int THREADS = kScan32Threads;
};

constexpr float kScan32RaiseLog2 = 8.f;   // the reference maximum is raised when a tile's maximum exceeds it by more (log2 units)

// BAL: the balanced split (the even split's instantiation has no segment loop)
template <int DK, int DV, bool BAL>
__global__ void __launch_bounds__(kScan32Threads, 1) __attribute__((amdgpu_waves_per_eu(2, 2))) k_scan32(const Scan32Args a) {
    using Cfg = Scan32Cfg<DK, DV>;
    using KLoader = DirectRowTile<Cfg::KROW, 1, Cfg::THREADS>;
    using VLoader = DirectRowTile<Cfg::VROW, 2, Cfg::THREADS>;
    constexpr int STEPS = Cfg::STEPS, MB = Cfg::MB, KT = Cfg::KT, KROW = Cfg::KROW, VROW = Cfg::VROW, STAGE = Cfg::STAGE;
    constexpr int KI = KLoader::ITERS, VI = VLoader::ITERS;     // load instructions per wavefront and tile
    extern __shared__ __align__(16) char smem[];
    __shared__ AncSet s_anc[kMaxT];
    __shared__ int s_par[kMaxT], s_depth[kMaxT], s_cmax[kMaxT];
    __shared__ int s_pref[kScan32MaxBalancedB + 1], s_wsum[kScan32Threads / 64];     // balanced split

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 31, hb = lane >> 5;

    const int n_pad = gridDim.x;
    const int wg = (blockIdx.x & 7) * (n_pad >> 3) + (blockIdx.x >> 3);   // every XCD gets a contiguous range of work
    if (wg >= a.n_wg) return;
    const int qg = wg % a.n_qg;

    // ---- segment-independent lane constants
    const uint32_t krow = (uint32_t)a.kc_s[2], vrow = (uint32_t)a.vc_s[2];
    KLoader kld;
    VLoader vld;
    kld.init(krow, tid);
    vld.init(vrow, tid);
    // this lane's byte offsets into a K tile for the four contraction steps of a 128-byte group: key row n of a
    // 32-key block, granule 2 q + hb, swizzled with bits 1..3 of the row
    int koff[4];
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) koff[q4] = n * KROW + KLoader::swizzled(n, 2 * q4 + hb) * 16;
    // this lane's byte offsets into a V tile for the transposing reads of column block mb: key row 4 hb + (p >> 2) of
    // a run of 16 keys, 8-byte chunk p & 3 of the 16 columns 32 mb + 16 mh .. (p = lane % 16, mh = bit 4 of the lane)
    int voff[MB];
    {
        const int p = lane & 15, mh = (lane >> 4) & 1, r = 4 * hb + (p >> 2);
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) voff[mb] = r * VROW + VLoader::swizzled(r, 4 * mb + 2 * mh) * 16 + (p & 3) * 8;
    }
    const int rr = wave * 32 + n;           // row of the workgroup
    const int jrow = rr / a.H_g;            // its verifier query within the group
    const float raise = kScan32RaiseLog2 / a.scale_log2;     // in raw score units

    // ---- this workgroup's work.  Even split: one segment.  Balanced split: the range [x, x_end) of the batch's cost
    //      sequence, walked pair by pair: pairs in (sequence, KV head) order, each costing its tiles plus pair_cost
    //      tile-equivalents for what every segment pays before and after its tiles (query rows, metadata, the first
    //      tile's latency, the state's write), which come first in the pair's interval; s_pref[b] = cost per KV head of the
    //      sequences before b.  A sequence counts ceil(n_cmp / 64) tiles, at least one if it has queries (so that every
    //      row gets its statistics written), and nothing at all if it has none.
    int x = 0, x_end = 1, range_len = 1, range_id = 0, b_cur = 0;
    const int pc = a.pair_cost;
    if constexpr (BAL) {
        auto cost_of = [&](int bb) {
            if (bb >= a.B) return 0;
            const int tq = a.n_query ? min(max(a.n_query[bb], 0), a.T) : a.T;
            return tq > 0 ? pc + max(1, (min(max(a.n_cmp[bb], 0), a.max_n_cmp) + kTile - 1) / kTile) : 0;
        };
        const int n0 = cost_of(2 * tid), n1 = cost_of(2 * tid + 1);
        int incl = n0 + n1;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int up = __shfl_up(incl, off);
            if (lane >= off) incl += up;
        }
        if (lane == 63) s_wsum[wave] = incl;
        __syncthreads();
        int before = 0;
        for (int w = 0; w < wave; ++w) before += s_wsum[w];
        const int excl = before + incl - (n0 + n1);
        if (tid == 0) s_pref[0] = 0;
        if (2 * tid < a.B) s_pref[2 * tid + 1] = excl + n0;
        if (2 * tid + 1 < a.B) s_pref[2 * tid + 2] = excl + n0 + n1;
        __syncthreads();
        const int W = s_pref[a.B] * a.H_kv;           // (the host keeps B * H_kv * cost of the longest below 2^30)
        range_len = max(max(1, a.range_min), (W + a.n_ranges - 1) / a.n_ranges);
        range_id = wg / a.n_qg;
        x = range_id * range_len;
        x_end = min(W, x + range_len);
        int lo = 0, hi = a.B;                         // the last sequence that starts at or before x: it holds position x
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (s_pref[mid] * a.H_kv <= x) lo = mid; else hi = mid;
        }
        b_cur = lo;

        // (written by the last range that has work, the one most likely to have time; by the first if the batch has none)
        if (a.imp_table && range_id == max(W - 1, 0) / range_len && qg == 0) {
            const int tiles2[2] = {n0 > 0 ? n0 - pc : 0, n1 > 0 ? n1 - pc : 0};     // tiles of this thread's two sequences
            block_build_work_table<kScan32Threads, 2>(tiles2, a.imp_items_max, 1 << 30, a.imp_table, s_wsum, tid);
        }
        if (x >= W) return;                           // (uniform) fewer ranges than workgroups
    }

    int b_meta = -1;            // the sequence whose metadata the LDS arrays hold
    SeqMeta sm{};
    do {
        int b, g, slot, seg_lo = 0, seg_hi = 0;
        bool finishes = false;                        // balanced: the segment holds the last tile of its pair
        if constexpr (BAL) {
            const int nb = s_pref[b_cur + 1] - s_pref[b_cur];          // > pair_cost: sequences without queries are stepped over
            const int off = x - s_pref[b_cur] * a.H_kv;
            b = b_cur;
            g = off / nb;
            const int c_lo = off - g * nb, c_hi = min(nb, c_lo + (x_end - x));     // in the pair's cost interval
            slot = range_id - (x - c_lo) / range_len;                  // ranges since the one that holds the pair's first position
            finishes = c_hi == nb;
            x += c_hi - c_lo;
            if (finishes && g == a.H_kv - 1) {
                ++b_cur;
                while (b_cur < a.B && s_pref[b_cur + 1] == s_pref[b_cur]) ++b_cur;
            }
            if (slot >= a.n_chunks) continue;                          // (cannot happen: range_len >= range_min)
            seg_lo = max(0, c_lo - pc);
            seg_hi = max(0, c_hi - pc);
            if (seg_hi == 0) {
                // the range ends before the pair's first tile: nothing to compute, the slot is marked empty (rows past
                // the sequence's query count exist in the workspace; nothing reads them)
                const int qi = qg * a.C + jrow;
                if (hb == 0 && jrow < a.C && qi < a.T) {
                    const int64_t grow = ((int64_t)b * a.T + qi) * a.H + g * a.H_g + rr % a.H_g;
                    *reinterpret_cast<float2*>(a.part_stats + ((int64_t)slot * a.rows_total + grow) * 2) = make_float2(0.f, 0.f);
                }
                continue;
            }
        } else {
            slot = (wg / a.n_qg) % a.n_chunks;
            const int bg = wg / (a.n_qg * a.n_chunks);
            b = bg / a.H_kv;
            g = bg % a.H_kv;
        }
        // The LDS ring and the metadata arrays of the previous segment are free after this barrier (its last tile waited
        // for every load).  Its state stores may still be in flight: they are older than every load of this segment, so
        // the counted waits below can only wait longer because of them.
        __syncthreads();

        // ---- B operands of S^T = K Q^T: row n of this wavefront's block of 32 rows, all contraction steps.  The address
        //      needs nothing from the sequence's metadata, so the loads go first (queries past the sequence's count exist in
        //      the buffer; rows that do not exist are zeroed below)
        u32x4 qf[STEPS];
        {
            const int qi = min(qg * a.C + jrow, a.T - 1);
            const char* qp = a.q + b * a.q_s[0] + qi * a.q_s[1] + (g * a.H_g + rr % a.H_g) * a.q_s[2] + hb * 16;
#pragma unroll
            for (int st = 0; st < STEPS; ++st) qf[st] = *reinterpret_cast<const u32x4*>(qp + st * 32);
        }

        if (!BAL || b != b_meta) {      // (uniform) the next KV head of the same sequence keeps the metadata
            sm = build_tree_meta(tid, b, a.T, a.seq_lens, a.n_query, a.n_cmp, a.parents, a.l, a.d, a.max_seq_len, a.max_n_cmp, s_par, s_depth,
                                 s_cmax, s_anc);
            b_meta = b;
        }
        const int nq_grp = min(a.C, sm.Tq - qg * a.C);    // verifier queries of this group that exist
        if (nq_grp <= 0) continue;                        // (uniform)

        // tiles of this slice, and how many leading tiles are visible in full to every row of the group
        int cm = 0, cmin = 0x7fffffff;
        for (int j = 0; j < nq_grp; ++j) {
            const int c = s_cmax[qg * a.C + j];
            cm = max(cm, c);
            cmin = min(cmin, c);
        }
        int t0, t1;
        if constexpr (BAL) {
            const int nt = (cm + kTile - 1) / kTile;      // this group's own tiles: at most the pair's
            t0 = min(seg_lo, nt);
            t1 = min(seg_hi, nt);
        } else {
            even_slice((cm + kTile - 1) / kTile, a.n_chunks, a.min_tiles, slot, t0, t1);
        }
        const int tf = cmin / kTile;            // tiles below tf need no mask

        const bool rvalid = jrow < nq_grp;
        const int qi_row = qg * a.C + (rvalid ? jrow : 0);
        const int cmaxr = rvalid ? s_cmax[qi_row] : 0;
        if (!rvalid) {
#pragma unroll
            for (int st = 0; st < STEPS; ++st) qf[st] = u32x4{0, 0, 0, 0};
        }

        // ---- tile loads: stage t = {K(t), V(t)} lives in slot (t - t0) % 3
        const __amdgpu_buffer_rsrc_t krsrc = KLoader::make_rsrc(a.kc + b * a.kc_s[0] + g * a.kc_s[1], (int64_t)sm.n_cmp * a.kc_s[2]);
        const __amdgpu_buffer_rsrc_t vrsrc = VLoader::make_rsrc(a.vc + b * a.vc_s[0] + g * a.vc_s[1], (int64_t)sm.n_cmp * a.vc_s[2]);
        auto stage_of = [&](int t) { return smem + ((t - t0) % 3) * STAGE; };
        auto issue_stage = [&](int t) {
            const int rows = min(kTile, sm.n_cmp - t * kTile);
            kld.template issue<true>(krsrc, (uint32_t)(t * kTile) * krow, stage_of(t), krow, rows, tid);
            vld.template issue<true>(vrsrc, (uint32_t)(t * kTile) * vrow, stage_of(t) + KT, vrow, rows, tid);
        };

        f32x16 acc[MB];
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[mb][i] = 0.f;
        float mref = -INFINITY, zrun = 0.f;

        if (t0 < t1) {
            issue_stage(t0);
            if (t0 + 1 < t1) issue_stage(t0 + 1);
        }
        for (int tile = t0; tile < t1; ++tile) {
            // Loads complete in issue order: stage `tile` has landed when no more loads are outstanding than the next
            // stage holds (stage tile + 2 is issued after this wait).
            if (tile + 1 < t1) wait_vmcnt<KI + VI>();
            else wait_vmcnt<0>();
            __syncthreads();        // stage `tile` is in LDS; every wavefront has left stage tile - 1
            if (tile + 2 < t1) issue_stage(tile + 2);
            __builtin_amdgcn_sched_barrier(0);
            const char* kt = stage_of(tile);
            const char* vt = kt + KT;

            // ---- S^T: s[kb] = keys 32 kb .. + 31 against this wavefront's rows; two independent accumulator chains.
            //      Lane layout: row n of the block, keys 32 kb + 8 j + 4 hb + r at vector index 4 j + r
            f32x16 s[2];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int i = 0; i < 16; ++i) s[kb][i] = 0.f;
            {
                // issue order, pinned: LEAD fragment reads ahead of their matrix instructions, so that the LDS latency of
                // every fragment is covered by the instructions of the fragments before it
                constexpr int N_RD = 2 * STEPS, LEAD = 6;
                auto k_frag = [&](int i) {      // fragment i: contraction step i / 2 of key block i % 2
                    const int st = i >> 1, kb = i & 1;
                    return lds_read16(kt + kb * 32 * KROW + koff[st & 3] + (st >> 2) * 128);
                };
                u32x4 kfb[LEAD];
#pragma unroll
                for (int i = 0; i < LEAD; ++i) kfb[i] = k_frag(i);
#pragma unroll
                for (int i = 0; i < N_RD; ++i) {
                    __builtin_amdgcn_sched_barrier(0);
                    s[i & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kfb[i % LEAD]), __builtin_bit_cast(bf16x8, qf[i >> 1]),
                                                                      s[i & 1], 0, 0, 0);
                    if (i + LEAD < N_RD) kfb[i % LEAD] = k_frag(i + LEAD);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            if (tile >= tf) {       // (uniform) visibility limits: keys at or beyond the row's limit become -inf
                const int lim = cmaxr - tile * kTile - 4 * hb;     // keys with 32 kb + 8 j + r < lim are visible
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int i = 0; i < 16; ++i)
                        if (32 * kb + 8 * (i >> 2) + (i & 3) >= lim) s[kb][i] = -INFINITY;
            }
            // ---- softmax step in the log2 domain: raise the reference if needed, scores -> bf16 probabilities (B operands:
            //      pk[kb][h] = keys 32 kb + 16 h .. + 15 in the order the products delivered them)
            float mx = max_nan(s[0][0], s[1][0]);
#pragma unroll
            for (int i = 1; i < 16; ++i) mx = max_nan(mx, max_nan(s[0][i], s[1][i]));
            mx = xor32_max(mx);
            const bool up = mx > mref + raise;
            const float m_new = up ? mx : mref;
            const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
            const float alpha = up ? fast_exp2((mref - m_use) * a.scale_log2) : 1.f;
            const float neg_ms = -m_use * a.scale_log2;
            float rs4[4] = {0.f, 0.f, 0.f, 0.f};      // four independent chains
            u32x4 pk[2][2];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
                float p[16];
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    p[i] = fast_exp2(__builtin_fmaf(s[kb][i], a.scale_log2, neg_ms));
                    rs4[i & 3] += p[i];
                }
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    bf16x8 v;
#pragma unroll
                    for (int e = 0; e < 8; ++e) v[e] = (__bf16)p[8 * h + e];
                    pk[kb][h] = __builtin_bit_cast(u32x4, v);
                }
            }
            const float rs = xor32_add((rs4[0] + rs4[1]) + (rs4[2] + rs4[3]));
            zrun = zrun * alpha + rs;
            mref = m_new;
            if (__builtin_amdgcn_ballot_w64(alpha != 1.f) != 0ull) {    // uniform; rare
#pragma unroll
                for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) acc[mb][i] *= alpha;
            }
            // ---- O^T += V^T P^T: A operand = 32 columns of V against 16 keys, read transposed from the row-major tile (two
            //      8-byte reads: keys 4 hb .. + 3 and 8 + 4 hb .. + 3 of the run, the order of the probabilities in pk)
            {
                constexpr int N_F = 4 * MB, LEAD = 4;       // fragment i: keys 16 (i / MB) .. + 15 against column block i % MB
                auto v_frag = [&](int i) {
                    const int kh = i / MB, mb = i % MB;
                    const u32x2 v0 = lds_read_tr16(vt + voff[mb] + (16 * kh) * VROW);
                    const u32x2 v1 = lds_read_tr16(vt + voff[mb] + (16 * kh + 8) * VROW);
                    return u32x4{v0[0], v0[1], v1[0], v1[1]};
                };
                u32x4 vfb[LEAD];
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int i = 0; i < LEAD; ++i) vfb[i] = v_frag(i);
#pragma unroll
                for (int i = 0; i < N_F; ++i) {
                    __builtin_amdgcn_sched_barrier(0);
                    const int kh = i / MB, mb = i % MB;
                    acc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vfb[i % LEAD]), __builtin_bit_cast(bf16x8, pk[kh >> 1][kh & 1]),
                                                                      acc[mb], 0, 0, 0);
                    if (i + LEAD < N_F) vfb[i % LEAD] = v_frag(i + LEAD);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }

        // ---- partial state of this slice: (reference maximum, Z) per row and the un-normalised accumulator; lane layout of
        //      acc[mb]: row n of the block, columns 32 mb + 8 j + 4 hb + r at vector index 4 j + r
        if (rvalid) {
            const int64_t grow = ((int64_t)b * a.T + qi_row) * a.H + g * a.H_g + rr % a.H_g;
            const int64_t pr = (int64_t)slot * a.rows_total + grow;
            if (hb == 0) {
                a.part_stats[pr * 2 + 0] = mref * a.scale_log2;   // statistics leave the kernel in the log2 domain
                a.part_stats[pr * 2 + 1] = zrun;
                // balanced split: the pair's last segment also marks the slots no range of this pair reached as empty
                if (finishes) {
                    for (int sl = slot + 1; sl < a.n_chunks; ++sl)
                        *reinterpret_cast<float2*>(a.part_stats + ((int64_t)sl * a.rows_total + grow) * 2) = make_float2(0.f, 0.f);
                }
            }
            if (zrun > 0.f) {
#pragma unroll
                for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        *reinterpret_cast<f32x4*>(a.part_acc + pr * DV + 32 * mb + 8 * j + 4 * hb) =
                            f32x4{acc[mb][4 * j], acc[mb][4 * j + 1], acc[mb][4 * j + 2], acc[mb][4 * j + 3]};
            }
        }
    } while (BAL && x < x_end);   // segments
}

}  // namespace ssv
