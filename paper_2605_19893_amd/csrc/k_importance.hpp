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
//
// Wide variant (RW = 2 or 4 row blocks of 64 per workgroup, for sequences with 128 / 256 and more routed rows per KV
// head): with one block of 64 rows per workgroup every workgroup streams the whole slice of k_cmp from L2 for its
// 64 rows, and at several hundred rows per KV head the pass is bound by that L2 traffic, not by its arithmetic.
// Here wavefront (rw, kw) holds the 64 rows of block rw as A operands, the ring is shared: every wavefront still
// fetches one strip of each tile, every strip is read by the RW wavefronts that hold different rows, and a wavefront
// works through RW strips of a tile.  K then reaches LDS once per 64 RW rows; one barrier per tile orders the fills
// of a ring slot against its readers.
#pragma once
#include "k_stream.hpp"
#include "work_table.hpp"

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
    const int32_t* work_table; // k_importance32: (sequence, slice, slices) per item (work_table.hpp), built earlier in the
                               // same call; null: every sequence is cut into n_imp_chunks slices
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
    static constexpr int DEPTH = 3;         // LDS slots per wavefront for K strips
    static constexpr int LDS_RING = 4 * DEPTH * KCH * 1024;   // dynamic LDS bytes
};


constexpr int kImpRows = 64;   // rows (routed queries x heads of the group) per workgroup

// HGM: 16 = one query per 16-row tile (H_g = 16); 4 = H_g of 4 or 8 (the four rows a lane holds in the result layout are
// heads of one query); 1 = H_g of 1 or 2.
// RW: blocks of 64 rows per workgroup (1, 2 or 4); wavefront w holds block w % RW and works on the strips
// (w / RW) RW .. + RW - 1 of every tile.
template <bool BF16, int DK, int HGM, int RW>
__global__ void __launch_bounds__(kThreads, 2) k_importance(const ImportanceArgs a) {
    using Cfg = ImportanceCfg<BF16, DK>;
    constexpr bool WIDE = HGM >= 4;
    constexpr int KCH = Cfg::KCH, RT = Cfg::RT, RC = WIDE ? 1 : 4, DEPTH = Cfg::DEPTH;
    constexpr int WGR = kImpRows * RW;        // rows per workgroup
    static_assert(RW == 1 || RW == 2 || RW == 4, "row blocks per workgroup");
    static_assert(DEPTH == 3 && 2 * KCH + 2 * RW < 64, "the waits below are written for three ring slots");
    extern __shared__ __align__(16) char smem[];   // [DEPTH][strip][KCH][1 KB]: the tiles in flight, one strip per wavefront
    // partial (M, Z) of every row, one per wavefront; with several row blocks it lives in the third ring slot, which
    // no strip enters before the first tile has been taken up (two workgroups per CU leave 80 KB each)
    __shared__ float2 s_part_own[RW == 1 ? 4 * WGR : 1];
    float2* s_part = RW == 1 ? s_part_own : reinterpret_cast<float2*>(smem + 2 * 4 * KCH * 1024);
    static_assert(4 * WGR * 8 <= 4 * KCH * 1024, "the partial statistics fit one ring slot");
    __shared__ __align__(16) float s_mp[WGR]; // M + log2 Z of every row: p = exp2(s - that)
    __shared__ AncSet s_anc[kMaxT];
    __shared__ int s_par[kMaxT], s_depth[kMaxT], s_cmax[kMaxT];
    __shared__ int s_qi[WGR];                 // verifier query behind every routed query of this workgroup

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 15, G = lane >> 4;
    const int rw = wave % RW, kw = wave / RW; // this wavefront's row block and its group of strips

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
            const int rr = rw * kImpRows + t * 16 + n;
            const int j = rr / a.H_g;
            // rows past the group's queries repeat its first query: whatever they produce is never stored, and
            // unconditional loads are not waited for here
            const int64_t qoff = b * a.q_s[0] + query_of(j < nq ? j : 0) * a.q_s[1] + (g * a.H_g + rr % a.H_g) * a.q_s[2];
#pragma unroll
            for (int kc = 0; kc < KCH; ++kc) qf[t][kc] = *reinterpret_cast<const u32x4*>(a.q + qoff + kc * 64 + G * 16);
        }
    };
    // Softmax statistics of the compressed scan: one row per lane and row block, every wavefront taking every fourth
    // slice; the loads of a batch of four slices are unconditional (clamped index) so that they are in flight together.
    // (one row block: the first batch is fetched together with the queries, before the sequence's metadata is
    // known; several: block by block at the merge, the registers are needed elsewhere)
    int64_t srow0 = 0;
    float2 st0[4];
    auto stats_row = [&](auto query_of, int nq, int rb) {
        const int rr = rb * kImpRows + lane;
        const int j = rr / a.H_g;
        return ((int64_t)b * a.T + query_of(j < nq ? j : 0)) * a.H + g * a.H_g + rr % a.H_g;
    };
    auto stats_load = [&](int s0, int64_t row, float2 (&st)[4]) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int sl = min(s0 + 4 * u, a.n_cmp_chunks - 1);
            st[u] = *reinterpret_cast<const float2*>(a.part_stats + ((int64_t)sl * a.rows_total + row) * 2);
        }
    };
    auto load_q_and_stats = [&](auto query_of, int nq) {
        load_q(query_of, nq);
        if constexpr (RW == 1) {
            srow0 = stats_row(query_of, nq, 0);
            stats_load(wave, srow0, st0);
        }
    };
    if (!a.share) {
        const auto query_of = [&](int j) { return qg * a.C + j; };
        load_q_and_stats(query_of, min(a.C, a.T - qg * a.C));
    }
    const SeqMeta sm = build_tree_meta(tid, b, a.T, a.seq_lens, a.n_query, a.n_cmp, a.parents, a.l, a.d, a.max_seq_len, a.max_n_cmp, s_par, s_depth,
                                       s_cmax, s_anc);
    const int Tq = sm.Tq;
    const int n_routed = a.share ? (Tq + a.share - 1) / a.share : Tq;
    const int nq_grp = min(a.C, n_routed - qg * a.C);
    if (nq_grp <= 0) return;
    if (tid < WGR) {
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

    // The strip this wavefront fetches: keys 16 wave + n of every tile, 16 bytes per 64-byte chunk and lane (B-operand
    // layout); rows past the last compressed row repeat it (their probabilities are masked by the visibility limit).
    // The strips go from global memory straight into a ring of DEPTH tile slots in LDS (buffer loads with the LDS
    // destination: lane-linear, so a lane of any wavefront that reads a strip finds at its own position the 16 bytes
    // of its key and granule), ahead of the tile in use: the registers are taken by the A operands.
    const __amdgpu_buffer_rsrc_t krsrc =
        DirectRowTile<Cfg::KROW>::make_rsrc(a.kc + b * a.kc_s[0] + g * a.kc_s[1], (int64_t)sm.n_cmp * a.kc_s[2]);
    const uint32_t krow = (uint32_t)a.kc_s[2];
    constexpr int STRIP = KCH * 1024, SLOT = 4 * STRIP;
    auto issue_strip = [&](int tile) {
        const uint32_t voff = (uint32_t)min(tile * kTile + 16 * wave + n, sm.n_cmp - 1) * krow + G * 16;
        char* dst = smem + ((tile - t0) % DEPTH) * SLOT + wave * STRIP;
#pragma unroll
        for (int kc = 0; kc < KCH; ++kc)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(krsrc, (__attribute__((address_space(3))) void*)(dst + kc * 1024), 16, (int)voff,
                                                     kc * 64, 0, 0);
    };
    // the first strips, the (shared-index variant) queries and the statistics below are all in flight together
#pragma unroll
    for (int i = 0; i < (RW == 1 ? DEPTH : DEPTH - 1); ++i)
        if (t0 + i < t1) issue_strip(t0 + i);
    if (a.share) {
        const auto query_of = [&](int j) { return s_qi[j]; };
        load_q_and_stats(query_of, nq_grp);
    }

    // merged statistics of every row of this workgroup: M = max_s m_s, Z = sum_s Z_s 2^(m_s - M)
    const int rows_wg = nq_grp * a.H_g;
#pragma unroll
    for (int rb = 0; rb < RW; ++rb) {
        const int rr = rb * kImpRows + lane;
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
        int64_t srow = srow0;
        if constexpr (RW > 1) {
            const int nq_all = a.share ? nq_grp : min(a.C, a.T - qg * a.C);
            srow = a.share ? stats_row([&](int j) { return s_qi[j]; }, nq_all, rb)
                           : stats_row([&](int j) { return qg * a.C + j; }, nq_all, rb);
            stats_load(wave, srow, st0);
        }
        merge4(wave, st0);
        for (int s0 = wave + 16; s0 < a.n_cmp_chunks; s0 += 16) {
            float2 st[4];
            stats_load(s0, srow, st);
            merge4(s0, st);
        }
        s_part[wave * WGR + rr] = make_float2(M, Z);
    }
    __syncthreads();
    if (wave < RW) {          // wavefront w finishes row block w
        const int rr = wave * kImpRows + lane;
        float Mn = -INFINITY;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const float2 o = s_part[u * WGR + rr];
            if (o.y > 0.f) Mn = fmaxf(Mn, o.x);
        }
        float Zt = 0.f;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const float2 o = s_part[u * WGR + rr];
            if (o.y > 0.f) Zt += o.y * fast_exp2(o.x - Mn);
        }
        s_mp[rr] = (rr < rows_wg && Zt > 0.f) ? Mn + __builtin_amdgcn_logf(Zt) : INFINITY;   // (the builtin is log2)
    }
    __syncthreads();

    // of the four rows (16 t + 4 G + r) this lane holds in the result layout: the softmax offset, the visibility
    // limit and the colsum row of their query
    float rowMp[RT][4];
    int rowC[RT][RC], rowQ[RT][RC];
#pragma unroll
    for (int t = 0; t < RT; ++t) {
        const float4 mp = *reinterpret_cast<const float4*>(s_mp + rw * kImpRows + t * 16 + 4 * G);
        rowMp[t][0] = mp.x; rowMp[t][1] = mp.y; rowMp[t][2] = mp.z; rowMp[t][3] = mp.w;
#pragma unroll
        for (int r = 0; r < RC; ++r) {
            const int j = (rw * kImpRows + t * 16 + 4 * G + r) / a.H_g;
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

    auto load_strip = [&](int tile, int strip, u32x4 (&kf)[KCH]) {
        const char* src = smem + ((tile - t0) % DEPTH) * SLOT + strip * STRIP + lane * 16;
#pragma unroll
        for (int kc = 0; kc < KCH; ++kc) kf[kc] = lds_read16(src + kc * 1024);
    };
    // One strip is 16 keys x 64 rows, in two halves: the scores (the matrix products), and the finish (exponentials,
    // head sums, stores).  The stores a finish issues are the same in every step (their predicates do not depend on
    // the tile: every key of a processed tile lies inside the colsum row).
    auto strip_scores = [&](const u32x4 (&kf)[KCH], f32x4 (&s)[RT]) {
#pragma unroll
        for (int t = 0; t < RT; ++t) s[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kc = 0; kc < KCH; ++kc)
#pragma unroll
            for (int t = 0; t < RT; ++t)
                s[t] = mma_frag<BF16>(qf[t][kc], kf[kc], s[t]);   // D[row 4G+r][key n]; rows past the group repeat its first query and are never stored
    };
    auto strip_finish = [&](int tile, int strip, const f32x4 (&s)[RT]) {
        const int c = tile * kTile + 16 * strip + n;
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

    // Software pipeline over the tiles of the slice, two levels deep.  (1) Strips are fetched three ahead of the
    // strip being finished, into the three ring slots.  (2) The matrix products of strip i + 1 are issued before the
    // exponentials and sums of strip i: the two are independent, so the matrix pipe works while the vector pipe
    // finishes the previous strip (in one wavefront, not only across the two wavefronts of a SIMD).
    // Loads and stores share one in-order counter: a strip has landed once no more operations are outstanding than
    // were issued after it: the KCH loads of each younger strip and the stores of the two steps since it was
    // issued (counting too few of them only waits longer).
    u32x4 kf[KCH];
    f32x4 s_cur[RT], s_next[RT];
    int tile = t0;
    if constexpr (RW == 1) {
        {
            const int young = min(2, t1 - t0 - 1);      // strips issued after the first one
            if (young == 2) wait_vmcnt<2 * KCH>();
            else if (young == 1) wait_vmcnt<KCH>();
            else wait_vmcnt<0>();
            load_strip(tile, wave, kf);
            strip_scores(kf, s_cur);
        }
        for (; tile + 3 < t1; ++tile) {
            issue_strip(tile + 3);                       // into the slot of strip `tile`, whose fragments are long consumed
            __builtin_amdgcn_sched_barrier(0);
            if (tile - t0 < 2) wait_vmcnt<2 * KCH>();
            else if (ns == 1) wait_vmcnt<2 * KCH + 2>();
            else wait_vmcnt_upto(2 * KCH + 2 * ns);
            load_strip(tile + 1, wave, kf);
            strip_scores(kf, s_next);
            strip_finish(tile, wave, s_cur);
#pragma unroll
            for (int t = 0; t < RT; ++t) s_cur[t] = s_next[t];
        }
        for (; tile + 1 < t1; ++tile) {                  // the last strips: nothing left to issue
            if (tile + 3 == t1) wait_vmcnt<KCH>();       // one younger strip (stores not counted: waits longer)
            else wait_vmcnt<0>();
            load_strip(tile + 1, wave, kf);
            strip_scores(kf, s_next);
            strip_finish(tile, wave, s_cur);
#pragma unroll
            for (int t = 0; t < RT; ++t) s_cur[t] = s_next[t];
        }
        strip_finish(tile, wave, s_cur);
    } else {
        // Shared ring, one barrier per tile.  Step `tile`: wait for the strip this wavefront fetched for it (younger
        // operations: the strip of the next tile, and the RW ns stores of each of the two steps since it was issued);
        // the barrier then says every strip of the tile has landed and every wavefront has left tile - 1, whose slot
        // the strip for tile + 2 may now overwrite.  Inside a tile the products of the next strip are issued before
        // the exponentials of the current one.
        for (; tile < t1; ++tile) {
            if (tile + 1 >= t1) wait_vmcnt<0>();
            else if (tile - t0 < 2) wait_vmcnt<KCH>();
            else wait_vmcnt_upto(KCH + 2 * RW * ns);
            __syncthreads();
            if (tile + 2 < t1) issue_strip(tile + 2);
            __builtin_amdgcn_sched_barrier(0);
            load_strip(tile, kw * RW, kf);
            strip_scores(kf, s_cur);
#pragma unroll
            for (int j = 0; j < RW; ++j) {
                if (j + 1 < RW) {
                    load_strip(tile, kw * RW + j + 1, kf);
                    strip_scores(kf, s_next);
                }
                strip_finish(tile, kw * RW + j, s_cur);
                if (j + 1 < RW) {
#pragma unroll
                    for (int t = 0; t < RT; ++t) s_cur[t] = s_next[t];
                }
            }
        }
    }
}

// ---- bf16 variant on the 32x32x16 matrix instruction ------------------------------------------------------------
// Measured on the device, independent v_mfma_f32_16x16x32_bf16 sustain about half of the chip's bf16 matrix peak
// and v_mfma_f32_32x32x16_bf16 all of it, so the bf16 pass takes its products in 32-row x 32-key blocks.
//   A operand = Q (lane l: row l % 32, the eight contraction elements 8 (l / 32) .. + 7 of a 16-element step),
//   B operand = K (lane l: key l % 32, same elements), result lane l: key l % 32, rows 8 j + 4 (l / 32) + r at
//   vector index 4 j + r: the rows of one lane are heads, so the head sum stays in the lane except for one exchange
//   between the two lane halves.
// A workgroup holds 64 RW rows; the 64-key tiles of its slice of k_cmp go from global memory straight into a ring of
// three swizzled row-major LDS tiles (fully coalesced loads shared by the whole workgroup, one barrier per tile);
// wavefront w works on RTW row tiles x KTW key tiles of every tile:
//   RW = 1: row tile w % 2, key tile w / 2;   RW = 2: row tile w, both key tiles;   RW = 4: row tiles 2w, 2w + 1, both key tiles.
template <int DK>
struct Importance32Cfg {
    static constexpr int KROW = DK * 2;
    static constexpr int STEPS = DK / 16;             // 16-element contraction steps
    static constexpr int DEPTH = 3;                   // tiles in the ring
    static constexpr int TILE = kTile * KROW;
    static constexpr int LDS_RING = DEPTH * TILE;
};

// NW: wavefronts per workgroup.  Eight (RW = 4 only) give every wavefront one row tile and both key tiles, four
// wavefronts per SIMD with two workgroups per CU: measured on the device, one wavefront issues a 32x32x16 matrix
// instruction every 64 clocks at best and its vector instructions at about half the rate a SIMD reaches with several
// wavefronts, so a tile step takes a wavefront the sum of its own matrix and vector work whatever else the SIMD holds;
// halving the work per wavefront halves the step, as long as the registers (128 per lane) allow four per SIMD.
template <int DK, int HGM, int RW, int NW = 4>
__global__ void __launch_bounds__(64 * NW, NW == 8 ? 1 : 2) __attribute__((amdgpu_waves_per_eu(NW == 8 ? 4 : 2, NW == 8 ? 4 : 8)))
k_importance32(const ImportanceArgs a) {
    using Cfg = Importance32Cfg<DK>;
    using Loader = DirectRowTile<Cfg::KROW, 1, 64 * NW>;
    static_assert(NW == 4 || (NW == 8 && RW == 4), "eight wavefronts: 256 rows only");
    constexpr int STEPS = Cfg::STEPS, DEPTH = Cfg::DEPTH, TILE = Cfg::TILE, LD = Loader::ITERS;
    constexpr int WGR = kImpRows * RW;                 // rows per workgroup
    constexpr int RTW = (RW == 4 && NW == 4) ? 2 : 1, KTW = RW == 1 ? 1 : 2;
    constexpr int QPT = HGM == 16 ? 1 : (HGM == 4 ? 4 : 16);   // stores per 32 x 32 block and lane (H_g = 8: two of the four are used)
    static_assert(RW == 1 || RW == 2 || RW == 4, "row blocks per workgroup");
    static_assert(4 * WGR * 8 <= TILE, "the partial statistics fit one ring slot");
    extern __shared__ __align__(16) char smem[];       // [DEPTH] tiles of 64 keys, swizzled row-major
    __shared__ __align__(16) float s_mp[WGR];          // M + log2 Z of every row: p = exp2(s - that)
    __shared__ AncSet s_anc[kMaxT];
    __shared__ int s_par[kMaxT], s_depth[kMaxT], s_cmax[kMaxT];
    __shared__ int s_qi[WGR];                          // verifier query behind every routed query of this workgroup
    // partial (M, Z) of every row, one per wavefront: in the third ring slot, which no tile enters before the first
    // tile has been taken up
    float2* s_part = reinterpret_cast<float2*>(smem + 2 * TILE);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 31, hb = lane >> 5;
    const int rt0 = RW == 1 ? (wave & 1) : wave * RTW; // first 32-row tile of this wavefront
    const int kt0 = RW == 1 ? (wave >> 1) : 0;         // first 32-key tile of this wavefront

    const int n_pad = gridDim.x;
    const int wg = (blockIdx.x & 7) * (n_pad >> 3) + (blockIdx.x >> 3);
    if (wg >= a.n_wg) return;
    const int qg = wg % a.n_qg;
    int chunk, n_chunks, b, g;
    if (a.work_table) {
        // a batch of mixed lengths: item = (sequence, slice), then KV head, then query group
        if (!work_table_item(a.work_table, wg / (a.n_qg * a.H_kv), a.B, b, chunk, n_chunks)) return;
        g = (wg / a.n_qg) % a.H_kv;
    } else {
        chunk = (wg / a.n_qg) % a.n_imp_chunks;
        n_chunks = a.n_imp_chunks;
        const int bg = wg / (a.n_qg * a.n_imp_chunks);
        b = bg / a.H_kv;
        g = bg % a.H_kv;
    }

    // A operands: row n of every row tile of this wavefront, all contraction steps.  When every query is routed the
    // rows are known before the sequence's metadata, and their loads overlap its latency (queries past the
    // sequence's count are loaded too, they exist in the buffer; nothing of theirs is used).
    u32x4 qf[RTW][STEPS];
    auto load_q = [&](auto query_of, int nq) {
#pragma unroll
        for (int t = 0; t < RTW; ++t) {
            const int rr = (rt0 + t) * 32 + n;
            const int j = rr / a.H_g;
            // rows past the group's queries repeat its first query: whatever they produce is never stored
            const int64_t qoff = b * a.q_s[0] + query_of(j < nq ? j : 0) * a.q_s[1] + (g * a.H_g + rr % a.H_g) * a.q_s[2];
#pragma unroll
            for (int st = 0; st < STEPS; ++st) qf[t][st] = *reinterpret_cast<const u32x4*>(a.q + qoff + st * 32 + hb * 16);
        }
    };
    if (!a.share) {
        const auto query_of = [&](int j) { return qg * a.C + j; };
        load_q(query_of, min(a.C, a.T - qg * a.C));
    }
    const SeqMeta sm = build_tree_meta(tid, b, a.T, a.seq_lens, a.n_query, a.n_cmp, a.parents, a.l, a.d, a.max_seq_len, a.max_n_cmp, s_par, s_depth,
                                       s_cmax, s_anc);
    const int Tq = sm.Tq;
    const int n_routed = a.share ? (Tq + a.share - 1) / a.share : Tq;
    const int nq_grp = min(a.C, n_routed - qg * a.C);
    if (nq_grp <= 0) return;
    if (tid < WGR) {
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
    even_slice(ntiles, n_chunks, 1, chunk, t0, t1);
    if (t0 >= t1) return;       // (uniform; cm > 0 from here on, so the sequence has compressed rows)

    // Tiles of 64 compressed rows, rows past the last one repeating it (their probabilities are masked by the
    // visibility limit), two tiles ahead of the one in use.
    const __amdgpu_buffer_rsrc_t krsrc = Loader::make_rsrc(a.kc + b * a.kc_s[0] + g * a.kc_s[1], (int64_t)sm.n_cmp * a.kc_s[2]);
    const uint32_t krow = (uint32_t)a.kc_s[2];
    Loader kdir;
    kdir.init(krow, tid);
    auto issue_tile = [&](int tile) {
        kdir.issue(krsrc, (uint32_t)(tile * kTile) * krow, smem + ((tile - t0) % DEPTH) * TILE, krow, min(kTile, sm.n_cmp - tile * kTile), tid);
    };
    issue_tile(t0);
    if (t0 + 1 < t1) issue_tile(t0 + 1);
    if (a.share) {
        const auto query_of = [&](int j) { return s_qi[j]; };
        load_q(query_of, nq_grp);
    }

    // merged statistics of every row of this workgroup: M = max_s m_s, Z = sum_s Z_s 2^(m_s - M); one row per lane and
    // block of 64 rows, every wavefront taking every fourth slice, four slices in flight
    const int rows_wg = nq_grp * a.H_g;
#pragma unroll
    for (int rb = 0; rb < RW; ++rb) {
        const int rr = rb * kImpRows + lane;
        const int j = rr / a.H_g;
        const int q_of_row = j < nq_grp ? s_qi[j] : s_qi[0];
        const int64_t srow = ((int64_t)b * a.T + q_of_row) * a.H + g * a.H_g + rr % a.H_g;
        float M = -INFINITY, Z = 0.f;
        if (wave >= 4) continue;      // (the first four wavefronts do this part, in the same order whatever NW is)
        for (int s0 = wave; s0 < a.n_cmp_chunks; s0 += 16) {
            float2 st[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int sl = min(s0 + 4 * u, a.n_cmp_chunks - 1);
                st[u] = *reinterpret_cast<const float2*>(a.part_stats + ((int64_t)sl * a.rows_total + srow) * 2);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                if (s0 + 4 * u < a.n_cmp_chunks && st[u].y > 0.f) {
                    const float Mn = fmaxf(M, st[u].x);
                    Z = Z * fast_exp2(M - Mn) + st[u].y * fast_exp2(st[u].x - Mn);
                    M = Mn;
                }
            }
        }
        s_part[wave * WGR + rr] = make_float2(M, Z);
    }
    __syncthreads();
    if (wave < RW) {          // wavefront w finishes row block w
        const int rr = wave * kImpRows + lane;
        float Mn = -INFINITY;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const float2 o = s_part[u * WGR + rr];
            if (o.y > 0.f) Mn = fmaxf(Mn, o.x);
        }
        float Zt = 0.f;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const float2 o = s_part[u * WGR + rr];
            if (o.y > 0.f) Zt += o.y * fast_exp2(o.x - Mn);
        }
        s_mp[rr] = (rr < rows_wg && Zt > 0.f) ? Mn + __builtin_amdgcn_logf(Zt) : INFINITY;   // (the builtin is log2)
    }
    __syncthreads();

    // of the sixteen rows (8 j + 4 hb + r) this lane holds of each of its row tiles: the softmax offset (in registers:
    // a 16-byte LDS read that all lanes of a half aim at one address is served as a bank conflict)
    float rowMp[RTW][16];
#pragma unroll
    for (int t = 0; t < RTW; ++t)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float4 mp = *reinterpret_cast<const float4*>(s_mp + (rt0 + t) * 32 + 8 * j + 4 * hb);
            rowMp[t][4 * j + 0] = mp.x; rowMp[t][4 * j + 1] = mp.y; rowMp[t][4 * j + 2] = mp.z; rowMp[t][4 * j + 3] = mp.w;
        }
    // the colsum row and the visibility limit behind each of this lane's stores of a block (H_g >= 4: kept in
    // registers; below that a block has up to sixteen queries per lane and they are looked up at the store)
    constexpr int NQR = HGM >= 4 ? QPT : 1;
    int rowC[RTW][NQR], rowQ[RTW][NQR];
    auto query_slot = [&](int row_in_wg, int& c_out, int& q_out) {
        const int j = row_in_wg / a.H_g;
        const bool ok = j < nq_grp;
        const int qi = s_qi[ok ? j : 0];
        c_out = ok ? s_cmax[qi] : 0;
        q_out = ok ? (b * a.T + qi) * a.H_kv + g : -1;
    };
    if constexpr (HGM >= 4) {
#pragma unroll
        for (int t = 0; t < RTW; ++t)
#pragma unroll
            for (int u = 0; u < QPT; ++u) {
                // H_g = 16: store u covers rows 16 u ..; this lane keeps query hb of the two.  H_g = 8: store u (0, 1)
                // covers queries 2 u and 2 u + 1, this lane keeps 2 u + hb.  H_g = 4: store u covers rows 8 u + 4 hb ...
                int row;
                if constexpr (HGM == 16) row = 16 * hb;
                else row = a.H_g == 8 ? (u < 2 ? 8 * (2 * u + hb) : -1) : 8 * u + 4 * hb;
                if (row < 0) { rowC[t][u] = 0; rowQ[t][u] = -1; }
                else query_slot((rt0 + t) * 32 + row, rowC[t][u], rowQ[t][u]);
            }
    }

    // this lane's byte offsets into a tile for the four contraction steps of a 128-byte group (the swizzle XORs the
    // granule index with bits 1..3 of the row, which for row 32 kt + n are those of n)
    int koff[4];
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) koff[q4] = n * Cfg::KROW + (((2 * q4 + hb) ^ ((n >> 1) & 7)) << 4);

    // The 32 x 32 blocks of one key tile, one per row tile of this wavefront: 16 scores per lane and block; every K
    // fragment read from LDS serves all RTW row tiles.  Then, per block: exponentials, head sums and stores.
    auto blocks_scores = [&](const char* tile_base, int kt, f32x16 (&s)[RTW]) {
#pragma unroll
        for (int t = 0; t < RTW; ++t)
#pragma unroll
            for (int i = 0; i < 16; ++i) s[t][i] = 0.f;
        const char* kb = tile_base + kt * 32 * Cfg::KROW;
#pragma unroll
        for (int st = 0; st < STEPS; ++st) {
            const u32x4 kf = lds_read16(kb + koff[st & 3] + (st >> 2) * 128);
#pragma unroll
            for (int t = 0; t < RTW; ++t)
                s[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, qf[t][st]), __builtin_bit_cast(bf16x8, kf), s[t], 0, 0, 0);
        }
    };
    auto block_finish = [&](int tile, int kt, int t, const f32x16& s) {
        const int c = tile * kTile + 32 * kt + n;
        float hs[4];                 // sums of this lane's four consecutive rows 8 j + 4 hb + 0..3
        float p[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) p[i] = fast_exp2(__builtin_fmaf(s[i], a.scale_log2, -rowMp[t][i]));
#pragma unroll
        for (int j = 0; j < 4; ++j) hs[j] = (p[4 * j] + p[4 * j + 1]) + (p[4 * j + 2] + p[4 * j + 3]);
        if constexpr (HGM == 16) {
            // rows 0..15 are one query, 16..31 the next; the exchange between the lane halves completes both sums and
            // leaves the first query's in the lower half, the second's in the upper half
            const float v0 = hs[0] + hs[1], v1 = hs[2] + hs[3];
            const auto f = __builtin_amdgcn_permlane32_swap(__float_as_uint(v0), __float_as_uint(v1), false, false);
            const float v = __uint_as_float(f[0]) + __uint_as_float(f[1]);
            if (rowQ[t][0] >= 0) a.colsum[(int64_t)rowQ[t][0] * a.nc_pitch + c] = c < rowC[t][0] ? v : 0.f;
        } else if constexpr (HGM == 4) {
            if (a.H_g == 8) {
                // rows 8 j .. 8 j + 7 are query j: half of it in each lane half
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    const auto f = __builtin_amdgcn_permlane32_swap(__float_as_uint(hs[2 * u]), __float_as_uint(hs[2 * u + 1]), false, false);
                    const float v = __uint_as_float(f[0]) + __uint_as_float(f[1]);
                    if (rowQ[t][u] >= 0) a.colsum[(int64_t)rowQ[t][u] * a.nc_pitch + c] = c < rowC[t][u] ? v : 0.f;
                }
            } else {
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    if (rowQ[t][u] >= 0) a.colsum[(int64_t)rowQ[t][u] * a.nc_pitch + c] = c < rowC[t][u] ? hs[u] : 0.f;
            }
        } else {
#pragma unroll
            for (int i = 0; i < 16; i += 2) {
                const int row = (rt0 + t) * 32 + 8 * (i >> 2) + 4 * hb + (i & 3);
                int c0, q0, c1, q1;
                query_slot(row, c0, q0);
                if (a.H_g == 2) {
                    if (q0 >= 0) a.colsum[(int64_t)q0 * a.nc_pitch + c] = c < c0 ? p[i] + p[i + 1] : 0.f;
                } else {
                    query_slot(row + 1, c1, q1);
                    if (q0 >= 0) a.colsum[(int64_t)q0 * a.nc_pitch + c] = c < c0 ? p[i] : 0.f;
                    if (q1 >= 0) a.colsum[(int64_t)q1 * a.nc_pitch + c] = c < c1 ? p[i + 1] : 0.f;
                }
            }
        }
    };
    // store instructions per block that are issued for certain (one whose predicate is false in every lane may or may
    // not be issued: it is not counted; counting too few only makes the waits below longer)
    int ns_step = 0;
    if constexpr (HGM >= 4) {
#pragma unroll
        for (int t = 0; t < RTW; ++t)
#pragma unroll
            for (int u = 0; u < QPT; ++u) ns_step += KTW * (__builtin_amdgcn_ballot_w64(rowQ[t][u] >= 0) != 0ull);
    }

    // Software pipeline over the tiles of the slice.  Step `tile`: wait for the loads this wavefront issued for it
    // (younger operations on the in-order counter: the LD loads of the next tile and the stores of the two steps
    // since); the barrier then says the whole tile has landed and every wavefront has left tile - 1, whose ring slot
    // the loads of tile + 2 may overwrite.  Inside a step the products of the next block are issued before the
    // exponentials of the current one, so the matrix pipe works while the vector pipe finishes a block.
    for (int tile = t0; tile < t1; ++tile) {
        if (tile + 1 >= t1) wait_vmcnt<0>();
        else if (tile - t0 < 2) wait_vmcnt<LD>();
        else wait_vmcnt_upto(LD + 2 * ns_step);
        __syncthreads();
        if (tile + 2 < t1) issue_tile(tile + 2);
        __builtin_amdgcn_sched_barrier(0);
        const char* tb = smem + ((tile - t0) % DEPTH) * TILE;
        f32x16 s_cur[RTW], s_next[RTW];
        blocks_scores(tb, kt0, s_cur);
#pragma unroll
        for (int k = 0; k < KTW; ++k) {
            if (k + 1 < KTW) blocks_scores(tb, kt0 + k + 1, s_next);
#pragma unroll
            for (int t = 0; t < RTW; ++t) block_finish(tile, kt0 + k, t, s_cur[t]);
            if (k + 1 < KTW) {
#pragma unroll
                for (int t = 0; t < RTW; ++t) s_cur[t] = s_next[t];
            }
        }
    }
}

}  // namespace ssv
