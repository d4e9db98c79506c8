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
//
// Work split: a workgroup holds the (at most 64) rows of its routed queries; every wavefront keeps ALL of
// them in registers as A operands and takes its own strip of 16 keys of every 64-key tile, whose K rows it streams
// from global memory, in B-operand layout, through a private ring of LDS slots (buffer loads with the LDS
// destination: the registers are taken by the A operands, and a lane reads back exactly the 16 bytes it
// fetched).  So no wavefront reads another's K from LDS (with 16 rows per wavefront every wavefront read the
// whole tile: four times the tile per step), the main loop has no barrier, and the head-summed probabilities go
// from registers to global memory.
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
    int64_t q_s[3];            // bytes: sequence, query, head
};

template <bool BF16, int DK>
struct ImportanceCfg {
    static constexpr int ES = BF16 ? 2 : 4;
    static constexpr int KROW = DK * ES;
    static constexpr int KCH = KROW / 64;
    static constexpr int RT = 4;            // 16-row tiles per workgroup: 64 rows
    static constexpr int DEPTH = 3;         // LDS slots per wavefront for K strips (DEPTH - 1 in flight)
    static constexpr int LDS_RING = 4 * DEPTH * KCH * 1024;   // dynamic LDS bytes
};


constexpr int kImpRows = 64;   // rows (routed queries x heads of the group) per workgroup

// HGM: 16 = one query per 16-row tile (H_g = 16); 4 = H_g of 4 or 8 (the four rows a lane holds in the result layout are
// heads of one query); 1 = H_g of 1 or 2.
template <bool BF16, int DK, int HGM>
__global__ void __launch_bounds__(kThreads, 2) k_importance(const ImportanceArgs a) {
    using Cfg = ImportanceCfg<BF16, DK>;
    constexpr bool WIDE = HGM >= 4;
    constexpr int ES = Cfg::ES, KCH = Cfg::KCH, RT = Cfg::RT, RC = WIDE ? 1 : 4, DEPTH = Cfg::DEPTH;
    static_assert(DEPTH == 3 && 2 * KCH + 2 < 64, "the waits below are written for two strips in flight");
    extern __shared__ __align__(16) char smem[];   // [wavefront][DEPTH][KCH][1 KB]: the strips in flight
    __shared__ float2 s_part[4 * kImpRows];   // partial (M, Z) of every row, one per wavefront
    __shared__ __align__(16) float s_mp[kImpRows];   // M + log2 Z of every row: p = exp2(s - that)
    __shared__ AncSet s_anc[kMaxT];
    __shared__ int s_par[kMaxT], s_depth[kMaxT], s_cmax[kMaxT];
    __shared__ int s_qi[kImpRows];              // verifier query behind every routed query of this workgroup

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 15, G = lane >> 4;

    const int n_pad = gridDim.x;
    const int wg = (blockIdx.x & 7) * (n_pad >> 3) + (blockIdx.x >> 3);
    if (wg >= a.n_wg) return;
    const int qg = wg % a.n_qg;
    const int chunk = (wg / a.n_qg) % a.n_imp_chunks;
    const int bg = wg / (a.n_qg * a.n_imp_chunks);
    const int b = bg / a.H_kv, g = bg % a.H_kv;

    // A operands: row n of every row tile of the workgroup, all 64-byte chunks.  When every query is routed the
    // rows are known before the sequence's metadata, and their loads overlap its latency (queries past the
    // sequence's count are loaded too, they exist in the buffer; nothing of theirs is used).
    u32x4 qf[RT][KCH];
    auto load_q = [&](auto query_of, int nq) {
#pragma unroll
        for (int t = 0; t < RT; ++t) {
            const int rr = t * 16 + n;
            const int j = rr / a.H_g;
            // rows past the group's queries repeat its first query: whatever they produce is never stored, and
            // unconditional loads are not waited for here
            const int64_t qoff = b * a.q_s[0] + query_of(j < nq ? j : 0) * a.q_s[1] + (g * a.H_g + rr % a.H_g) * a.q_s[2];
#pragma unroll
            for (int kc = 0; kc < KCH; ++kc) qf[t][kc] = *reinterpret_cast<const u32x4*>(a.q + qoff + kc * 64 + G * 16);
        }
    };
    // Softmax statistics of the compressed scan: one row per lane, every wavefront taking every fourth slice; the
    // loads of a batch of four slices are unconditional (clamped index) so that they are in flight together.
    int64_t srow = 0;
    float2 st0[4];
    auto stats_row = [&](auto query_of, int nq) {
        const int j = lane / a.H_g;
        return ((int64_t)b * a.T + query_of(j < nq ? j : 0)) * a.H + g * a.H_g + lane % a.H_g;
    };
    auto stats_load = [&](int s0, float2 (&st)[4]) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int sl = min(s0 + 4 * u, a.n_cmp_chunks - 1);
            st[u] = *reinterpret_cast<const float2*>(a.part_stats + ((int64_t)sl * a.rows_total + srow) * 2);
        }
    };
    if (!a.share) {
        const auto query_of = [&](int j) { return qg * a.C + j; };
        const int nq = min(a.C, a.T - qg * a.C);
        load_q(query_of, nq);
        srow = stats_row(query_of, nq);
        stats_load(wave, st0);
    }
    const SeqMeta sm = build_tree_meta(tid, b, a.T, a.seq_lens, a.n_query, a.n_cmp, a.parents, a.l, a.d, a.max_seq_len, a.max_n_cmp, s_par, s_depth,
                                       s_cmax, s_anc);
    const int Tq = sm.Tq;
    const int n_routed = a.share ? (Tq + a.share - 1) / a.share : Tq;
    const int nq_grp = min(a.C, n_routed - qg * a.C);
    if (nq_grp <= 0) return;
    if (tid < kImpRows) {
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
    if (t0 >= t1) return;       // (uniform; cm > 0 from here on, so the sequence has compressed rows)

    // This wavefront's strip: keys 16 wave + n of every tile, 16 bytes per 64-byte chunk and lane (B-operand layout);
    // rows past the last compressed row repeat it (their probabilities are masked by the visibility limit).  The
    // strips go from global memory straight into a ring of DEPTH wavefront-private LDS slots (buffer loads with
    // the LDS destination: lane-linear, so every lane later reads back exactly the 16 bytes it fetched), DEPTH - 1
    // strips ahead of the one in use: the registers are taken by the A operands.
    const __amdgpu_buffer_rsrc_t krsrc =
        DirectRowTile<Cfg::KROW>::make_rsrc(a.kc + b * a.kc_s[0] + g * a.kc_s[1], (int64_t)sm.n_cmp * a.kc_s[2]);
    const uint32_t krow = (uint32_t)a.kc_s[2];
    char* ring = smem + wave * (DEPTH * KCH * 1024);
    auto issue_strip = [&](int tile) {
        const uint32_t voff = (uint32_t)min(tile * kTile + 16 * wave + n, sm.n_cmp - 1) * krow + G * 16;
        char* dst = ring + ((tile - t0) % DEPTH) * (KCH * 1024);
#pragma unroll
        for (int kc = 0; kc < KCH; ++kc)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(krsrc, (__attribute__((address_space(3))) void*)(dst + kc * 1024), 16, (int)voff,
                                                     kc * 64, 0, 0);
    };
    // the first strips, the (shared-index variant) queries and the statistics below are all in flight together
#pragma unroll
    for (int i = 0; i < DEPTH - 1; ++i)
        if (t0 + i < t1) issue_strip(t0 + i);
    if (a.share) {
        const auto query_of = [&](int j) { return s_qi[j]; };
        load_q(query_of, nq_grp);
        srow = stats_row(query_of, nq_grp);
        stats_load(wave, st0);
    }

    // merged statistics of every row of this workgroup: M = max_s m_s, Z = sum_s Z_s 2^(m_s - M)
    const int rows_wg = nq_grp * a.H_g;
    {
        const int rr = lane;
        const bool ok = rr < rows_wg;
        float M = -INFINITY, Z = 0.f;
        auto merge4 = [&](int s0, const float2 (&st)[4]) {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                if (s0 + 4 * u < a.n_cmp_chunks && st[u].y > 0.f) {
                    const float Mn = fmaxf(M, st[u].x);
                    Z = Z * fast_exp2(M - Mn) + st[u].y * fast_exp2(st[u].x - Mn);
                    M = Mn;
                }
            }
        };
        merge4(wave, st0);
        for (int s0 = wave + 16; s0 < a.n_cmp_chunks; s0 += 16) {
            float2 st[4];
            stats_load(s0, st);
            merge4(s0, st);
        }
        s_part[wave * kImpRows + rr] = make_float2(M, Z);
        __syncthreads();
        if (wave == 0) {
            float Mn = -INFINITY;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const float2 o = s_part[u * kImpRows + rr];
                if (o.y > 0.f) Mn = fmaxf(Mn, o.x);
            }
            float Zt = 0.f;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const float2 o = s_part[u * kImpRows + rr];
                if (o.y > 0.f) Zt += o.y * fast_exp2(o.x - Mn);
            }
            s_mp[rr] = (ok && Zt > 0.f) ? Mn + __builtin_amdgcn_logf(Zt) : INFINITY;   // (the builtin is log2)
        }
    }
    __syncthreads();

    // of the four rows (16 t + 4 G + r) this lane holds in the result layout: the softmax offset, the visibility
    // limit and the colsum row of their query
    float rowMp[RT][4];
    int rowC[RT][RC], rowQ[RT][RC];
#pragma unroll
    for (int t = 0; t < RT; ++t) {
        const float4 mp = *reinterpret_cast<const float4*>(s_mp + t * 16 + 4 * G);
        rowMp[t][0] = mp.x; rowMp[t][1] = mp.y; rowMp[t][2] = mp.z; rowMp[t][3] = mp.w;
#pragma unroll
        for (int r = 0; r < RC; ++r) {
            const int j = (t * 16 + 4 * G + r) / a.H_g;
            const bool ok = j < nq_grp;
            const int qi = s_qi[ok ? j : 0];
            rowC[t][r] = ok ? s_cmax[qi] : 0;
            rowQ[t][r] = ok ? (b * a.T + qi) * a.H_kv + g : -1;
        }
    }
    // HGM == 16: lane group G ends up with the head sum of row tile (= query) G
    int myC = 0, myQ = -1;
    if constexpr (HGM == 16) {
#pragma unroll
        for (int t = 0; t < RT; ++t)
            if (G == t) { myC = rowC[t][0]; myQ = rowQ[t][0]; }     // (the same in every lane for a given t)
    }

    auto load_strip = [&](int tile, u32x4 (&kf)[KCH]) {
        const char* src = ring + ((tile - t0) % DEPTH) * (KCH * 1024) + lane * 16;
#pragma unroll
        for (int kc = 0; kc < KCH; ++kc) kf[kc] = lds_read16(src + kc * 1024);
    };
    // One strip: 16 keys x 64 rows.  The stores it issues are the same in every step (their predicates do not
    // depend on the tile: every key of a processed tile lies inside the colsum row).
    auto strip_step = [&](int tile, const u32x4 (&kf)[KCH]) {
        f32x4 s[RT];
#pragma unroll
        for (int t = 0; t < RT; ++t) s[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kc = 0; kc < KCH; ++kc)
#pragma unroll
            for (int t = 0; t < RT; ++t)
                s[t] = mma_frag<BF16>(qf[t][kc], kf[kc], s[t]);   // D[row 4G+r][key n]; rows past the group repeat its first query and are never stored
        const int c = tile * kTile + 16 * wave + n;
        if constexpr (WIDE) {
            float hs[RT];     // head sums of this lane's four rows of each row tile (one query), unmasked
#pragma unroll
            for (int t = 0; t < RT; ++t) {
                float p[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) p[r] = fast_exp2(__builtin_fmaf(s[t][r], a.scale_log2, -rowMp[t][r]));
                hs[t] = (p[0] + p[1]) + (p[2] + p[3]);
            }
            if constexpr (HGM == 16) {
                // Sum over the four lane groups and hand row tile t to lane group t in one butterfly: the swap of
                // (x, y) leaves x's pair of 16-lane rows in the even rows and y's in the odd ones (lower and upper
                // 32 lanes for the second stage).
                const auto e01 = __builtin_amdgcn_permlane16_swap(__float_as_uint(hs[0]), __float_as_uint(hs[1]), false, false);
                const auto e23 = __builtin_amdgcn_permlane16_swap(__float_as_uint(hs[2]), __float_as_uint(hs[3]), false, false);
                const float r01 = __uint_as_float(e01[0]) + __uint_as_float(e01[1]);
                const float r23 = __uint_as_float(e23[0]) + __uint_as_float(e23[1]);
                const auto f = __builtin_amdgcn_permlane32_swap(__float_as_uint(r01), __float_as_uint(r23), false, false);
                const float v = __uint_as_float(f[0]) + __uint_as_float(f[1]);
                if (myQ >= 0) a.colsum[(int64_t)myQ * a.nc_pitch + c] = c < myC ? v : 0.f;
            } else {
                const int gpq = a.H_g >> 2;                     // lane groups per query: 1 or 2
#pragma unroll
                for (int t = 0; t < RT; ++t) {
                    float v = hs[t];
                    if (gpq == 2) v = xor16_add(v);
                    if ((G % gpq) == 0 && rowQ[t][0] >= 0) a.colsum[(int64_t)rowQ[t][0] * a.nc_pitch + c] = c < rowC[t][0] ? v : 0.f;
                }
            }
        } else {
#pragma unroll
            for (int t = 0; t < RT; ++t) {
                float p[4];
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    p[r] = c < rowC[t][r] ? fast_exp2(__builtin_fmaf(s[t][r], a.scale_log2, -rowMp[t][r])) : 0.f;
                if (a.H_g == 2) {
                    if (rowQ[t][0] >= 0) a.colsum[(int64_t)rowQ[t][0] * a.nc_pitch + c] = p[0] + p[1];
                    if (rowQ[t][2] >= 0) a.colsum[(int64_t)rowQ[t][2] * a.nc_pitch + c] = p[2] + p[3];
                } else {
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        if (rowQ[t][r] >= 0) a.colsum[(int64_t)rowQ[t][r] * a.nc_pitch + c] = p[r];
                }
            }
        }
    };
    // store instructions per step that are issued for certain (a store whose predicate is false in every lane may or
    // may not be issued: it is not counted)
    int ns = 0;
    if constexpr (HGM == 16) {
        ns = 1;      // lane group 0 always has a query
    } else if constexpr (WIDE) {
        const int gpq = a.H_g >> 2;
#pragma unroll
        for (int t = 0; t < RT; ++t) ns += __builtin_amdgcn_ballot_w64((G % gpq) == 0 && rowQ[t][0] >= 0) != 0ull;
    } else {
#pragma unroll
        for (int t = 0; t < RT; ++t)
#pragma unroll
            for (int r = 0; r < 4; ++r)
                if (a.H_g == 1 || !(r & 1)) ns += __builtin_amdgcn_ballot_w64(rowQ[t][r] >= 0) != 0ull;
    }

    // Software pipeline over the tiles of the slice.  Loads and stores share one in-order counter: the strip of a
    // tile has landed once no more operations are outstanding than were issued after it: the KCH loads of each
    // younger strip and the stores of the two steps since it was issued (counting too few of them only waits
    // longer).
    auto step = [&](int tile) {
        u32x4 kf[KCH];
        load_strip(tile, kf);
        strip_step(tile, kf);
    };
    int tile = t0;
    for (; tile + 2 < t1; ++tile) {
        issue_strip(tile + 2);
        __builtin_amdgcn_sched_barrier(0);
        if (tile - t0 < 2) wait_vmcnt<2 * KCH>();
        else if (ns == 1) wait_vmcnt<2 * KCH + 2>();
        else wait_vmcnt_upto(2 * KCH + 2 * ns);
        step(tile);
    }
    if (tile + 1 < t1) {
        wait_vmcnt<KCH>();
        step(tile);
        ++tile;
    }
    wait_vmcnt<0>();
    step(tile);
}

}  // namespace ssv
