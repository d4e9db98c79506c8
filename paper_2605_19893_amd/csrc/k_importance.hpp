// Routing, part 2 (Section 5.1: the routing launch scores the importance of blocks): the compressed
// probabilities of every head must be normalised with that head's global softmax statistics before
// they are summed over the heads of a GQA group, so this pass runs after the compressed scan has
// produced the per-slice (max, sum) pairs.  It recomputes S = Q K_cmp^T for its slice of compressed
// rows (k_cmp only, no v_cmp), forms p = exp2(s - M) / Z with the merged statistics, adds the heads
// of each query, and writes colsum[b, i, g, c] = sum_{h in g} p_h[c].
//
// The kernel works on a list of routed queries: every verifier query in the exact variant, only the
// representative of each group of `share` queries in the approximate shared-index variant (Section 4.3).
//
// The tile product is taken in the orientation D[query row][key] (Q as the A operand): a lane then
// holds four heads of one key, so the head sum is three in-register adds plus at most two
// cross-lane exchanges.
#pragma once
#include "k_stream.hpp"

namespace ssv {

struct ImportanceArgs {
    const char *q, *kc;
    const int32_t *seq_lens, *n_cmp, *n_query, *parents;
    const float* part_stats;   // slots [0, n_cmp_chunks) hold the compressed-scan partial statistics
    float* colsum;             // [B, T, H_kv, nc_pitch]
    int B, T, H, H_kv, H_g;
    int C, n_qg;               // routed queries per workgroup; workgroups over the routed queries of a sequence
    int share;                 // 0: every query is routed; > 0: one representative per group of `share` queries
    int l, d;
    int max_seq_len, max_n_cmp;   // host-side bounds the lengths read from device memory are clamped to
    float scale_log2;
    int n_cmp_chunks;          // slices of the compressed scan (partial statistics to merge)
    int n_imp_chunks;          // slices of this kernel's own pass over k_cmp
    int n_wg;
    int nc_pitch;
    int64_t rows_total;
    int64_t kc_s[3];           // bytes
};

template <bool BF16, int DK>
struct ImportanceCfg {
    static constexpr int ES = BF16 ? 2 : 4;
    static constexpr int KROW = DK * ES;
    static constexpr int KP = KROW + 16;
    static constexpr int KCH = KROW / 64;
    static constexpr int LDS_K = kTile * KP;
    // LDS bytes: K tile, merged row statistics, per-sequence tree metadata and routed-query list, then the
    // head-summed tile [C][64]
    static constexpr int lds_bytes(int C) { return LDS_K + 256 * 8 + kMaxT * 32 + 64 + C * kTile * 4; }
};

template <bool BF16, int DK, int NRT>
__global__ void __launch_bounds__(kThreads, 2) k_importance(const ImportanceArgs a) {
    using Cfg = ImportanceCfg<BF16, DK>;
    constexpr int ES = Cfg::ES, KP = Cfg::KP, KCH = Cfg::KCH;
    extern __shared__ __align__(16) char smem[];
    char* sK = smem;
    float2* s_stat = reinterpret_cast<float2*>(sK + Cfg::LDS_K);   // [128] (M, 1/Z) per workgroup row
    AncSet* s_anc = reinterpret_cast<AncSet*>(s_stat + 256);
    int* s_par = reinterpret_cast<int*>(s_anc + kMaxT);
    int* s_depth = s_par + kMaxT;
    int* s_cmax = s_depth + kMaxT;
    int* s_qi = s_cmax + kMaxT;                                    // verifier query behind every routed query of this workgroup
    float* s_cs = reinterpret_cast<float*>(s_qi + kMaxT + 16);     // [C][64] head-summed probabilities

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 15, G = lane >> 4;

    const int n_pad = gridDim.x;
    const int wg = (blockIdx.x & 7) * (n_pad >> 3) + (blockIdx.x >> 3);
    if (wg >= a.n_wg) return;
    const int qg = wg % a.n_qg;
    const int chunk = (wg / a.n_qg) % a.n_imp_chunks;
    const int bg = wg / (a.n_qg * a.n_imp_chunks);
    const int b = bg / a.H_kv, g = bg % a.H_kv;

    const SeqMeta sm = build_tree_meta(tid, b, a.T, a.seq_lens, a.n_query, a.n_cmp, a.parents, a.l, a.d, a.max_seq_len, a.max_n_cmp, s_par, s_depth,
                                       s_cmax,
                                       s_anc);
    const int L = sm.L, Tq = sm.Tq;
    const int n_routed = a.share ? (Tq + a.share - 1) / a.share : Tq;
    const int nq_grp = min(a.C, n_routed - qg * a.C);
    if (nq_grp <= 0) return;
    if (tid < a.C) {
        int qi = 0;
        if (tid < nq_grp) {
            const int r = qg * a.C + tid;
            qi = a.share ? group_representative(s_depth, r * a.share, min((r + 1) * a.share, Tq)) : r;
        }
        s_qi[tid] = qi;
    }
    __syncthreads();

    int cm = 0;
    for (int j = 0; j < nq_grp; ++j) cm = max(cm, s_cmax[s_qi[j]]);
    const int ntiles = (cm + kTile - 1) / kTile;
    int t0, t1;
    even_slice(ntiles, a.n_imp_chunks, 1, chunk, t0, t1);
    if (t0 >= t1) return;

    // merged softmax statistics of every row of this workgroup: M = max_s m_s, Z = sum_s Z_s 2^(m_s - M).
    // Two threads per row, each taking every other slice; the loads of a batch of eight slices are
    // unconditional (clamped index) so that they are in flight together.
    const int rows_wg = nq_grp * a.H_g;
    {
        const int rr = tid & 127, half = tid >> 7;
        const bool ok = rr < rows_wg;
        const int64_t grow = ((int64_t)b * a.T + s_qi[ok ? rr / a.H_g : 0]) * a.H + g * a.H_g + rr % a.H_g;
        float M = -INFINITY, Z = 0.f;
        for (int s0 = half; s0 < a.n_cmp_chunks; s0 += 16) {
            float2 st[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int sl = min(s0 + 2 * u, a.n_cmp_chunks - 1);
                st[u] = *reinterpret_cast<const float2*>(a.part_stats + ((int64_t)sl * a.rows_total + grow) * 2);
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                if (s0 + 2 * u < a.n_cmp_chunks && st[u].y > 0.f) {
                    const float Mn = fmaxf(M, st[u].x);
                    Z = Z * fast_exp2(M - Mn) + st[u].y * fast_exp2(st[u].x - Mn);
                    M = Mn;
                }
            }
        }
        float2* s_half = s_stat + 128;     // second half of the pair, merged below
        if (half) s_half[rr] = make_float2(M, Z);
        __syncthreads();
        if (!half) {
            const float2 o = s_half[rr];
            const float Mn = fmaxf(M, o.x);
            float Zt = 0.f;
            if (Z > 0.f) Zt += Z * fast_exp2(M - Mn);
            if (o.y > 0.f) Zt += o.y * fast_exp2(o.x - Mn);
            s_stat[rr] = make_float2(Zt > 0.f ? Mn : 0.f, (ok && Zt > 0.f) ? 1.f / Zt : 0.f);
        }
    }

    // A operand: this lane's query rows (row n of each row tile), all 64-byte chunks
    u32x4 qf[NRT][KCH];
#pragma unroll
    for (int t = 0; t < NRT; ++t) {
        const int rr = (wave + 4 * t) * 16 + n;
        const int j = rr / a.H_g;
        const bool ok = j < nq_grp;
        const int64_t grow = ((int64_t)b * a.T + s_qi[ok ? j : 0]) * a.H + g * a.H_g + rr % a.H_g;
#pragma unroll
        for (int kc = 0; kc < KCH; ++kc) {
            qf[t][kc] = u32x4{0, 0, 0, 0};
            if (ok) qf[t][kc] = *reinterpret_cast<const u32x4*>(a.q + grow * (DK * ES) + kc * 64 + G * 16);
        }
    }
    __syncthreads();

    // statistics and visibility limits of the four rows (4 G + r) this lane holds in the result layout
    float rowM[NRT][4], rowIZ[NRT][4];
    int rowC[NRT][4];
#pragma unroll
    for (int t = 0; t < NRT; ++t)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int rr = (wave + 4 * t) * 16 + 4 * G + r;
            const int j = rr / a.H_g;
            const bool ok = j < nq_grp;
            const float2 st = s_stat[ok ? rr : 0];
            rowM[t][r] = st.x;
            rowIZ[t][r] = ok ? st.y : 0.f;
            rowC[t][r] = ok ? s_cmax[s_qi[j]] : 0;
        }

    const char* kbase = a.kc + b * a.kc_s[0] + g * a.kc_s[1];
    RowTileRegs<Cfg::KROW> kregs;     // the loads of the next tile are in flight while this one is computed
    kregs.init((uint32_t)a.kc_s[2], tid);
    kregs.issue(kbase + (int64_t)t0 * kTile * a.kc_s[2], (uint32_t)a.kc_s[2], min(kTile, sm.n_cmp - t0 * kTile), tid);
    for (int tile = t0; tile < t1; ++tile) {
        const int base = tile * kTile;
        __syncthreads();
        kregs.template commit<KP>(sK, min(kTile, sm.n_cmp - base), tid);
        __syncthreads();
        if (tile + 1 < t1)
            kregs.issue(kbase + (int64_t)(base + kTile) * a.kc_s[2], (uint32_t)a.kc_s[2], min(kTile, sm.n_cmp - base - kTile), tid);
#pragma unroll
        for (int t = 0; t < NRT; ++t) {
            const int rt = wave + 4 * t;
            if (rt * 16 >= rows_wg) continue;
#pragma unroll
            for (int kt = 0; kt < 4; ++kt) {
                f32x4 s = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int kc = 0; kc < KCH; ++kc) {
                    const u32x4 kf = lds_read16(sK + (16 * kt + n) * KP + kc * 64 + G * 16);
                    s = mma_frag<BF16>(qf[t][kc], kf, s);   // D[row 4G+r][key n]
                }
                const int c = base + 16 * kt + n;
                float p[4];
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    p[r] = c < rowC[t][r] ? fast_exp2(s[r] * a.scale_log2 - rowM[t][r]) * rowIZ[t][r] : 0.f;
                // head sum; rows 16 rt + 4 G + r, H_g heads per query
                const int key = 16 * kt + n;
                if (a.H_g >= 4) {
                    float v = (p[0] + p[1]) + (p[2] + p[3]);
                    if (a.H_g >= 8) v = xor16_add(v);
                    if (a.H_g >= 16) v = xor32_add(v);
                    const int gpq = a.H_g >> 2;                  // lane groups per query
                    if ((G % gpq) == 0) {
                        const int j = (rt * 16 + 4 * G) / a.H_g;
                        if (j < nq_grp) s_cs[j * kTile + key] = v;
                    }
                } else if (a.H_g == 2) {
                    const int j = (rt * 16 + 4 * G) >> 1;
                    if (j < nq_grp) s_cs[j * kTile + key] = p[0] + p[1];
                    if (j + 1 < nq_grp) s_cs[(j + 1) * kTile + key] = p[2] + p[3];
                } else {
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int j = rt * 16 + 4 * G + r;
                        if (j < nq_grp) s_cs[j * kTile + key] = p[r];
                    }
                }
            }
        }
        __syncthreads();
        for (int i = tid; i < nq_grp * kTile; i += kThreads) {
            const int j = i / kTile, key = i % kTile;
            if (base + key < a.nc_pitch)
                a.colsum[(((int64_t)b * a.T + s_qi[j]) * a.H_kv + g) * a.nc_pitch + base + key] = s_cs[i];
        }
    }
}

}  // namespace ssv
