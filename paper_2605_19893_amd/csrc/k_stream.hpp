// Streaming attention kernel: one workgroup = one (sequence, KV head, group of C verifier queries)
// and one slice of one branch's key tiles.  The three NSA branches (Section 2.2) are three mask
// policies over the same tile loop:
//   CMP  rows of k_cmp / v_cmp, visible while the compressed window is complete for the query;
//   WIN  raw KV tiles covering the union of the group's sliding windows, masked per row by the
//        query's own absolute position and tree ancestry (Section 4.1: shared window scan with
//        per-query local masks);
//   SLC  raw KV tiles of the merged schedule: the sorted, de-duplicated union of the group's
//        selected block indices with a query->block ownership mask; every block is loaded once
//        and logits of non-owning rows are masked to -inf (Section 4.2).
// Each workgroup writes one partial softmax state (running max, sum, un-normalised P.V) per row;
// the combine kernel merges the slices of a branch and applies the gates.
//
// Matrix tiles: S^T = K . Q^T with K rows as the MFMA M dimension, so that each lane ends up
// with four consecutive keys of one query row; P^T then is directly the B operand of
// O^T = V^T . P^T without a round trip through LDS.
#pragma once
#include "device_common.hpp"
#include "k_topn.hpp"
#include "work_table.hpp"

namespace ssv {

struct StreamArgs {
    const char *q, *k, *v, *kc, *vc;
    const int32_t *seq_lens, *n_cmp, *n_query, *parents, *sel_idx;
    float *part_stats, *part_acc;
    int B, T, H, H_kv, H_g, C, n_qg;
    int l, d, n_sel, w;
    int max_seq_len, max_n_cmp;   // host-side bounds the lengths read from device memory are clamped to
    float scale_log2;
    int n_cmp_chunks, n_win_splits, n_slc_splits, min_tiles;
    int slot_lo, slot_cnt;   // partial-state slots computed by this launch
    const int32_t* cmp_table; // launches with the compressed scan: its work table (below), or null
    int cmp_items_max;       // capacity of that table in items
    int joint;               // <WIN|SLC> launch: > 0 = parts per group over window tiles and schedule entries together (below)
    int n_wg;                // real workgroups (the grid is padded to a multiple of 8)
    int max_sched, bitmap_words;
    int64_t rows_total;
    int64_t k_s[3], v_s[3], kc_s[3], vc_s[3];   // strides in bytes: sequence, KV head, row
    int64_t q_s[3];                             // strides in bytes: sequence, query, head
    // selected-branch launch of the refresh path that also does the top-n selection (fused_topn != 0): every
    // workgroup selects for the queries of its group from the head-summed probabilities, one query per wavefront,
    // and the first slice of each group writes the sets out
    const float* colsum;     // [B, T, H_kv, nc_pitch]
    int32_t* sel_out;        // [B, T, H_kv, n_sel]
    int fused_topn, nc_pitch, l_sel, n_init, n_local, max_blocks, share;
};

// LDS the fused selection needs (it uses the tile buffers, which are idle until the schedule exists)
__host__ __device__ inline size_t fused_topn_lds_bytes(int max_blocks, int C, int n_sel) {
    return 4 * wave_topn_lds_bytes(max_blocks) + (size_t)C * n_sel * 4;
}

template <bool BF16, int DK, int DV>
struct StreamCfg {
    static constexpr int ES = BF16 ? 2 : 4;
    static constexpr int KROW = DK * ES;            // bytes per K row
    static constexpr int LDS_KD = kTile * KROW;     // one K tile in LDS (unpadded, granules swizzled); there are two
    static constexpr int KCH = KROW / 64;           // 64-byte chunks per K row
    static constexpr int VP = kTile * ES + 16;      // fp32: LDS pitch of a V^T row (64 keys)
    static constexpr int VR = DV * ES + 32;         // bf16: LDS pitch of a V row (the tile stays row-major)
    static constexpr int MT = DV / 16;              // 16-row tiles of O^T
    static constexpr int LDS_K = 2 * LDS_KD;
    static constexpr int LDS_VT = BF16 ? kTile * VR : DV * VP;
};

__host__ __device__ inline size_t stream_lds_bytes(size_t lds_k, size_t lds_vt, int max_sched, int bitmap_words) {
    size_t n = lds_k + lds_vt;
    n += (size_t)max_sched * 8;          // ownership masks
    n += (size_t)max_sched * 4;          // block ids
    n += (size_t)bitmap_words * 4 * 2;   // bitmap + prefix
    n += kMaxT * 16 + kMaxT * 4 * 3 + kTile * 4 + 16; // anc, par, depth, cmax, key positions, scalars
    return (n + 15) & ~(size_t)15;
}

enum Role { ROLE_CMP = 0, ROLE_WIN = 1, ROLE_SLC = 2 };

// Slice `part` of `parts` over n items, sizes differing by at most one; fewer slices are used when
// they would fall below min_items each (the surplus slices are empty).
__device__ __forceinline__ void even_slice(int n, int parts, int min_items, int part, int& lo, int& hi) {
    const int used = max(1, min(parts, n / max(1, min_items)));
    if (part >= used) { lo = hi = 0; return; }
    lo = part * n / used;          // part <= 64 and n <= 2^14 tiles: no overflow
    hi = (part + 1) * n / used;
}

// ROLES: which branches this instantiation can run (bit 0 CMP, bit 1 WIN, bit 2 SLC).  The refresh path
// launches <CMP|WIN> and then <SLC>, the reuse path launches all three at once, the unfused execution launches
// each branch on its own, and <WIN|SLC> follows the matrix-core scan of the compressed cache (k_scan32.hpp); code of
// absent roles is compiled out.
//
// Work table of the compressed scan (cmp_table, batches of mixed lengths; work_table.hpp): the scan's workgroups come
// first in the launch, cmp_items_max * H_kv * n_qg of them, and take (sequence, slice, slices) from the table: slices per
// sequence in proportion to its length, all of about the same length.  Slice j of a sequence owns compressed slot j;
// the last slice marks the slots beyond the sequence's slices as empty.  The workgroups of the other branches follow,
// cut as always.  Workgroup ids go round-robin over the XCDs here (the groups of one slice stay together): the slices
// are equally long, so an equal count per XCD is what balances them.
//
// Joint slicing (the <WIN|SLC> launch, joint = P > 0): the window tiles of a group and the entries of its merged schedule
// form one list, window first, cut into P even parts; a workgroup takes one part, which may end the window and begin
// the schedule.  It writes one state per branch: part j owns window slot j and selected slot j (slots
// [n_cmp_chunks, + P) and [n_cmp_chunks + P, + P)); the state of a branch its part does not touch is marked empty.
// Separate slices per branch leave the window's workgroup (9 tiles at w = 512) idle while the schedule's
// (up to 32 tiles each) run on.
constexpr int kRolesCmp = 1, kRolesWin = 2, kRolesCmpWin = 3, kRolesSlc = 4, kRolesWinSlc = 6, kRolesAll = 7;

// Two workgroups per CU (the LDS of the full-size shapes allows no more), stated to the compiler as exactly two
// waves per SIMD: left free to aim for three, it trades away the read-ahead of the K fragments for registers that
// no third wave can use.

template <bool BF16, int DK, int DV, int NRT, int ROLES>
__global__ void __launch_bounds__(kThreads, 2) __attribute__((amdgpu_waves_per_eu(2, 2))) k_stream(const StreamArgs a) {
    using Cfg = StreamCfg<BF16, DK, DV>;
    constexpr int ES = Cfg::ES, KROWB = Cfg::KROW, KCH = Cfg::KCH, VP = Cfg::VP, VR = Cfg::VR, MT = Cfg::MT;
    extern __shared__ __align__(16) char smem[];
    char* sK0 = smem;                  // two K tiles: the global->LDS loads of tile i+1 land while tile i is read
    char* sVT = sK0 + Cfg::LDS_K;
    uint64_t* s_own = reinterpret_cast<uint64_t*>(sVT + Cfg::LDS_VT);
    AncSet* s_anc = reinterpret_cast<AncSet*>(s_own + a.max_sched);
    int* s_id = reinterpret_cast<int*>(s_anc + kMaxT);
    uint32_t* s_bitmap = reinterpret_cast<uint32_t*>(s_id + a.max_sched);
    uint32_t* s_prefix = s_bitmap + a.bitmap_words;
    int* s_par = reinterpret_cast<int*>(s_prefix + a.bitmap_words);
    int* s_depth = s_par + kMaxT;
    int* s_cmax = s_depth + kMaxT;
    int* s_kpos = s_cmax + kMaxT;      // [64] key positions of the current tile (16-byte aligned)
    int* s_scalar = s_kpos + kTile;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 15, G = lane >> 4;

    // XCD-aware order: consecutive dispatch ids go round-robin over the 8 XCDs, so give every XCD a
    // contiguous range of logical work items; the query groups of one (sequence, head, slice), which
    // read the same tiles, are adjacent in logical order and therefore share an L2.
    const int n_pad = gridDim.x;
    int wg, qg, slot, b, g;
    int cmp_parts = 0;            // work table: slices of this sequence's compressed rows (0: the launch-wide count)
    bool from_table = false;
    if constexpr (ROLES & 1) from_table = a.cmp_table != nullptr;     // (uniform for the launch)
    if (from_table) {
        // the n_qg groups of a slice stay adjacent on one XCD, consecutive slices go to consecutive XCDs
        const int x = blockIdx.x & 7, j = blockIdx.x >> 3;
        wg = ((j / a.n_qg) * 8 + x) * a.n_qg + j % a.n_qg;
        if (wg >= a.n_wg) return;
        qg = wg % a.n_qg;
        const int n_tab = a.cmp_items_max * a.H_kv * a.n_qg;
        if (wg < n_tab) {
            g = (wg / a.n_qg) % a.H_kv;
            if (!work_table_item(a.cmp_table, wg / (a.n_qg * a.H_kv), a.B, b, slot, cmp_parts)) return;
            slot = min(max(slot, 0), a.n_cmp_chunks - 1);
        } else {
            const int rest = a.slot_cnt - a.n_cmp_chunks, w2 = wg - n_tab;      // the other branches' slots of this launch
            slot = a.slot_lo + a.n_cmp_chunks + (w2 / a.n_qg) % rest;
            const int bg = w2 / (a.n_qg * rest);
            b = bg / a.H_kv;
            g = bg % a.H_kv;
        }
    } else {
        wg = (blockIdx.x & 7) * (n_pad >> 3) + (blockIdx.x >> 3);
        if (wg >= a.n_wg) return;
        qg = wg % a.n_qg;
        slot = a.slot_lo + (wg / a.n_qg) % a.slot_cnt;
        const int bg = wg / (a.n_qg * a.slot_cnt);
        b = bg / a.H_kv;
        g = bg % a.H_kv;
    }

    const bool joint = ROLES == kRolesWinSlc && a.joint > 0;    // (uniform for the launch)
    int role, part;
    if (joint) { role = ROLE_SLC; part = slot - a.slot_lo; }     // (the role of the first segment is set below)
    else if (slot < a.n_cmp_chunks) { role = ROLE_CMP; part = slot; }
    else if (slot < a.n_cmp_chunks + a.n_win_splits) { role = ROLE_WIN; part = slot - a.n_cmp_chunks; }
    else { role = ROLE_SLC; part = slot - a.n_cmp_chunks - a.n_win_splits; }
    const bool r_cmp = (ROLES & 1) && role == ROLE_CMP;
    bool r_win = (ROLES & 2) && role == ROLE_WIN;
    bool r_slc = (ROLES & 4) && role == ROLE_SLC;      // joint: true up to the schedule's construction, then per segment

    // ---- query fragments (B operand of S^T = K Q^T), kept in registers for the whole slice.  Their addresses need
    //      nothing from the sequence's metadata, so the loads go first and overlap the latency of everything below
    //      (rows past the sequence's query count exist in the buffer; their fragments are zeroed once the count is known)
    //      (two row tiles per wave: the registers do not allow it; those launches are long, the loads follow the metadata)
    u32x4 qf[NRT][KCH];
    if constexpr (NRT == 1) {
        const int rr = wave * 16 + n;
        const int qi = min(qg * a.C + rr / a.H_g, a.T - 1);
        const char* qp = a.q + b * a.q_s[0] + qi * a.q_s[1] + (g * a.H_g + rr % a.H_g) * a.q_s[2] + G * 16;
#pragma unroll
        for (int kc = 0; kc < KCH; ++kc) qf[0][kc] = *reinterpret_cast<const u32x4*>(qp + kc * 64);
    }
    // (reuse mode, selected branch) this thread's first entry of the group's index sets, fetched early for the same reason
    int pre_id = -1;
    if constexpr (ROLES & 4) {
        if (r_slc && !a.fused_topn && tid < a.C * a.n_sel && qg * a.C + tid / a.n_sel < a.T)
            pre_id = a.sel_idx[(((int64_t)b * a.T + qg * a.C + tid / a.n_sel) * a.H_kv + g) * a.n_sel + tid % a.n_sel];
    }

    const SeqMeta sm = build_tree_meta(tid, b, a.T, a.seq_lens, a.n_query, a.n_cmp, a.parents, a.l, a.d, a.max_seq_len, a.max_n_cmp, s_par, s_depth,
                                       s_cmax,
                                       s_anc);
    const int L = sm.L, Tq = sm.Tq;
    const int nq_grp = min(a.C, Tq - qg * a.C);   // verifier queries of this group that exist
    const int n_slots_kv = L + Tq;                // raw KV rows that exist for this sequence

    // ---- per-lane row metadata
    bool rvalid[NRT];
    AncSet anc[NRT];
    int pos[NRT], cmax[NRT], iq[NRT];
    int64_t grow[NRT];
#pragma unroll
    for (int t = 0; t < NRT; ++t) {
        const int rr = (wave + 4 * t) * 16 + n;
        iq[t] = rr / a.H_g;
        const int qi = qg * a.C + iq[t];
        rvalid[t] = iq[t] < nq_grp;
        const int qs = rvalid[t] ? qi : 0;
        anc[t] = rvalid[t] ? s_anc[qs] : AncSet{0ull, 0ull};
        pos[t] = L + s_depth[qs];
        cmax[t] = rvalid[t] ? s_cmax[qs] : 0;
        grow[t] = ((int64_t)b * a.T + qs) * a.H + g * a.H_g + rr % a.H_g;
    }

    // ---- fused top-n selection (Section 5.1: routing, then attention over the selected blocks)
    int32_t* s_sel = nullptr;     // [C][n_sel] index sets of the group's queries, in the (still idle) tile buffers
    if constexpr (ROLES == kRolesSlc || ROLES == kRolesWinSlc) {
        if (a.fused_topn && r_slc) {      // (uniform per workgroup)
            s_sel = reinterpret_cast<int32_t*>(smem + 4 * wave_topn_lds_bytes(a.max_blocks));
            const WaveTopnScratch ws = wave_topn_scratch(smem + wave * wave_topn_lds_bytes(a.max_blocks), a.max_blocks);
            for (int j = wave; j < a.C; j += 4) {
                const int x = qg * a.C + j;
                if (x >= a.T) break;
                int32_t* out = s_sel + j * a.n_sel;
                if (x >= Tq) {
                    if (lane < a.n_sel) out[lane] = -1;
                } else {
                    // the approximate shared-index variant selects for the representative of the query's sharing group
                    const int i = a.share ? group_representative(s_depth, (x / a.share) * a.share, min((x / a.share + 1) * a.share, Tq)) : x;
                    wave_topn(a.colsum + (((int64_t)b * a.T + i) * a.H_kv + g) * a.nc_pitch, min(s_cmax[i], a.nc_pitch),
                              min((L + i) / a.l_sel, a.max_blocks - 1), a.l, a.d, a.l_sel, a.n_sel, a.n_init, a.n_local, ws, lane, out);
                }
                wave_lds_sync();
                if (part == 0 && lane < a.n_sel) a.sel_out[(((int64_t)b * a.T + x) * a.H_kv + g) * a.n_sel + lane] = out[lane];
            }
            __syncthreads();
        }
    }

    // ---- tile range of this workgroup
    int t0 = 0, t1 = 0;           // CMP / WIN: tile indices; SLC: schedule entries
    int jw0 = 0, jw1 = 0, js0 = 0, js1 = 0;      // joint slicing: both ranges
    if (nq_grp > 0) {
        if (r_cmp) {
            int cm = 0;
            for (int j = 0; j < nq_grp; ++j) cm = max(cm, s_cmax[qg * a.C + j]);
            const int ntiles = (cm + kTile - 1) / kTile;
            even_slice(ntiles, cmp_parts ? cmp_parts : a.n_cmp_chunks, a.min_tiles, part, t0, t1);
        } else if (r_win) {
            int dmin = 1 << 30;
            for (int j = 0; j < nq_grp; ++j) dmin = min(dmin, s_depth[qg * a.C + j]);
            const int wlo = max(0, L + dmin - a.w + 1) / kTile;
            const int whi = (n_slots_kv + kTile - 1) / kTile;
            even_slice(whi - wlo, a.n_win_splits, a.min_tiles, part, t0, t1);
            t0 += wlo;
            t1 += wlo;
        } else if (r_slc) {
            // merged schedule: bitmap over blocks -> ranks by prefix popcount -> sorted unique list + ownership
            const int nblk = min((n_slots_kv + kTile - 1) / kTile, a.bitmap_words * 32);
            const int nwords = (nblk + 31) >> 5;
            for (int i = tid; i < nwords; i += kThreads) s_bitmap[i] = 0;
            for (int i = tid; i < a.max_sched; i += kThreads) s_own[i] = 0ull;
            __syncthreads();
            const int n_ent = nq_grp * a.n_sel;
            for (int i = tid; i < n_ent; i += kThreads) {
                const int j = i / a.n_sel, e = i % a.n_sel;
                const int id = s_sel ? s_sel[i] : (i < kThreads ? pre_id : a.sel_idx[(((int64_t)b * a.T + qg * a.C + j) * a.H_kv + g) * a.n_sel + e]);
                if (id >= 0 && id < nblk) atomicOr(&s_bitmap[id >> 5], 1u << (id & 31));
            }
            __syncthreads();
            if (wave == 0) {
                const int per = (nwords + 63) >> 6;
                const int w0 = lane * per, w1 = min(nwords, w0 + per);
                int cnt = 0;
                for (int i = w0; i < w1; ++i) cnt += __popc(s_bitmap[i]);
                int incl = cnt;
#pragma unroll
                for (int off = 1; off < 64; off <<= 1) {
                    const int up = __shfl_up(incl, off);
                    if (lane >= off) incl += up;
                }
                int run = incl - cnt;
                for (int i = w0; i < w1; ++i) { s_prefix[i] = run; run += __popc(s_bitmap[i]); }
                if (lane == 63) s_scalar[0] = incl;
            }
            __syncthreads();
            for (int i = tid; i < n_ent; i += kThreads) {
                const int j = i / a.n_sel, e = i % a.n_sel;
                const int id = s_sel ? s_sel[i] : (i < kThreads ? pre_id : a.sel_idx[(((int64_t)b * a.T + qg * a.C + j) * a.H_kv + g) * a.n_sel + e]);
                if (id >= 0 && id < nblk) {
                    const uint32_t wd = s_bitmap[id >> 5];
                    const int rank = s_prefix[id >> 5] + __popc(wd & ((1u << (id & 31)) - 1u));
                    s_id[rank] = id;
                    atomicOr(reinterpret_cast<unsigned long long*>(&s_own[rank]), 1ull << j);
                }
            }
            __syncthreads();
            const int len = s_scalar[0];
            if (!joint) even_slice(len, a.n_slc_splits, a.min_tiles, part, t0, t1);
            else {
                // this part of [window tiles | schedule entries]: its window tiles [jw0, jw1), its entries [js0, js1)
                int dmin = 1 << 30;
                for (int j = 0; j < nq_grp; ++j) dmin = min(dmin, s_depth[qg * a.C + j]);
                const int wlo = max(0, L + dmin - a.w + 1) / kTile;
                const int nw = (n_slots_kv + kTile - 1) / kTile - wlo;
                int lo, hi;
                even_slice(nw + len, a.joint, a.min_tiles, part, lo, hi);
                jw0 = wlo + min(lo, nw);
                jw1 = wlo + min(hi, nw);
                js0 = max(lo, nw) - nw;
                js1 = max(hi, nw) - nw;
            }
        }
    }

    // ---- fragments of rows that do not exist are zero (nothing of theirs is ever written; zero keeps their
    //      scores finite)
#pragma unroll
    for (int t = 0; t < NRT; ++t) {
        if constexpr (NRT > 1) {
            const int64_t qoff = b * a.q_s[0] + (qg * a.C + iq[t]) * a.q_s[1] + (g * a.H_g + ((wave + 4 * t) * 16 + n) % a.H_g) * a.q_s[2];
#pragma unroll
            for (int kc = 0; kc < KCH; ++kc) {
                qf[t][kc] = u32x4{0, 0, 0, 0};
                if (rvalid[t]) qf[t][kc] = *reinterpret_cast<const u32x4*>(a.q + qoff + kc * 64 + G * 16);
            }
        } else if (!rvalid[t]) {
#pragma unroll
            for (int kc = 0; kc < KCH; ++kc) qf[t][kc] = u32x4{0, 0, 0, 0};
        }
    }

    f32x4 acc[NRT][MT];
    float mrun[NRT], zrun[NRT];

    const char* kbase;
    const char* vbase;
    int64_t krow, vrow;
    if (r_cmp) {
        kbase = a.kc + b * a.kc_s[0] + g * a.kc_s[1];
        vbase = a.vc + b * a.vc_s[0] + g * a.vc_s[1];
        krow = a.kc_s[2];
        vrow = a.vc_s[2];
    } else {
        kbase = a.k + b * a.k_s[0] + g * a.k_s[1];
        vbase = a.v + b * a.v_s[0] + g * a.v_s[1];
        krow = a.k_s[2];
        vrow = a.v_s[2];
    }
    const int rows_exist = r_cmp ? sm.n_cmp : n_slots_kv;
    // bf16: this lane's address into the row-major V tile for the transposing reads: key row 4 G + (n >> 2) of each
    // run of 16 keys, 8-byte chunk (n & 3) of each 16-column tile
    const int vt_rb = (4 * G + (n >> 2)) * VR + (n & 3) * 8;

    // Software pipeline: the global loads of tile it+1 are issued before tile it is computed.  K goes straight into
    // the other of two LDS tiles (no registers, no LDS stores); V is staged in registers for one tile step (LDS has
    // no room for a second V tile at two workgroups per CU) and stored to LDS at the start of its own step.  Two
    // barriers per tile separate the LDS writes from the fragment reads.  Measured with in-kernel clocks, the
    // prefetched loads have nearly always arrived by the time they are needed at one tile ahead.
    constexpr int AHEAD = 1;
    const __amdgpu_buffer_rsrc_t krsrc = DirectRowTile<Cfg::KROW>::make_rsrc(kbase, (int64_t)max(rows_exist, 0) * krow);
    DirectRowTile<Cfg::KROW> kdir;
    TransposedTileRegs<BF16, DV> vregs[AHEAD];
    auto tile_of = [&](int it) { return r_slc ? s_id[it] : it; };
    auto issue_tile = [&](int it, TransposedTileRegs<BF16, DV>& vr) {
        const int base_n = tile_of(it) * kTile;
        const int vr_n = min(kTile, rows_exist - base_n);
        kdir.issue(krsrc, (uint32_t)base_n * (uint32_t)krow, sK0 + ((it - t0) & 1) * Cfg::LDS_KD, (uint32_t)krow, vr_n, tid);
        vr.issue(vbase + (int64_t)base_n * vrow, (uint32_t)vrow, vr_n, tid);
    };
    kdir.init((uint32_t)krow, tid);
#pragma unroll
    for (int j = 0; j < AHEAD; ++j) vregs[j].init((uint32_t)vrow, tid);
    // this lane's two base offsets into a K tile (row n of a 16-key tile, granule G of an even / odd 64-byte chunk)
    const int k_rb_e = DirectRowTile<Cfg::KROW>::read_base(n, G, 0), k_rb_o = DirectRowTile<Cfg::KROW>::read_base(n, G, 1);
    // wave-wide bounds for the "every key of the tile is valid for every row" fast path (rows that do not
    // exist are don't-cares: nothing of theirs is ever written)
    int full_cmax = 0x7fffffff, full_lo = -0x7fffffff;
#pragma unroll
    for (int t = 0; t < NRT; ++t) {
        if (rvalid[t]) { full_cmax = min(full_cmax, cmax[t]); full_lo = max(full_lo, pos[t] - a.w + 1); }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        full_cmax = min(full_cmax, __shfl_xor(full_cmax, off));
        full_lo = max(full_lo, __shfl_xor(full_lo, off));
    }
    // One tile; vcur holds the V rows of tile `it` and, once committed to LDS, takes those of tile it + AHEAD.
    auto tile_step = [&](const int it, TransposedTileRegs<BF16, DV>& vcur) {
        const char* sK = sK0 + ((it - t0) & 1) * Cfg::LDS_KD;
        const int tile = tile_of(it);
        const uint64_t own = r_slc ? s_own[it] : ~0ull;
        const int base = tile * kTile;
        const int valid_rows = min(kTile, rows_exist - base);
        const bool has_drafts = !r_cmp && base + kTile > L;   // uniform: the tile holds draft slots

        if (it > t0) __syncthreads();   // every wave has finished reading the previous tile
        if constexpr (BF16) vcur.template commit_rows<VR>(sVT, valid_rows, tid);
        else vcur.template commit<VP>(sVT, valid_rows, tid);
        if (has_drafts && tid < kTile) {   // absolute position of every key of the tile (tree drafts: L + depth)
            const int s = base + tid;
            s_kpos[tid] = s < L ? s : (s - L < Tq ? L + s_depth[s - L] : 0x7fffffff);
        }
        __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): this wavefront's global->LDS loads of the K tile have landed
        __syncthreads();
        if (it + AHEAD < t1) issue_tile(it + AHEAD, vcur);
        __builtin_amdgcn_sched_barrier(0);    // the loads stay ahead of the compute below (they have been seen to sink past it)

        // ---- validity of this lane's 16 keys (4 key tiles x 4 registers) for each of its query rows;
        //      bit 4 kt + r <-> key base + 16 kt + 4 G + r
        uint32_t vm[NRT];
        const bool tile_full = (r_cmp && base + kTile <= full_cmax) || (r_win && !has_drafts && base >= full_lo);   // uniform
#pragma unroll
        for (int t = 0; t < NRT; ++t) {
            vm[t] = 0xFFFFu;
            if (tile_full) continue;
            vm[t] = 0;
            if (!rvalid[t]) continue;
            if (r_cmp) {
                const int lim = cmax[t] - base - 4 * G;          // keys with 16 kt + r < lim are visible
#pragma unroll
                for (int kt = 0; kt < 4; ++kt) vm[t] |= ((1u << min(max(lim - 16 * kt, 0), 4)) - 1u) << (4 * kt);
            } else if (r_win || (r_slc && ((own >> iq[t]) & 1ull))) {
                if (!has_drafts) {                               // every key is a committed token
                    if (r_slc) vm[t] = 0xFFFFu;
                    else {
                        const int lo = pos[t] - a.w + 1 - base - 4 * G;   // keys with 16 kt + r >= lo are in the window
#pragma unroll
                        for (int kt = 0; kt < 4; ++kt)
                            vm[t] |= (0xFu & ~((1u << min(max(lo - 16 * kt, 0), 4)) - 1u)) << (4 * kt);
                    }
                } else {
                    // visibility of the tile's 64 slots as one bit mask: committed slots, then the ancestor bits
                    const int cl = L - base;      // committed slots at the front of the tile (< 64 here; may be <= 0)
                    uint64_t vis;                 // (uniform branches: cl is the same for the whole workgroup)
                    if (cl > 0) vis = ((1ull << cl) - 1ull) | (anc[t].lo << cl);
                    else if (cl == 0) vis = anc[t].lo;
                    else if (cl > -64) vis = (anc[t].lo >> (-cl)) | (anc[t].hi << (64 + cl));
                    else if (cl == -64) vis = anc[t].hi;
                    else vis = cl > -128 ? anc[t].hi >> (-cl - 64) : 0ull;
#pragma unroll
                    for (int kt = 0; kt < 4; ++kt) vm[t] |= (uint32_t)((vis >> (16 * kt + 4 * G)) & 0xFull) << (4 * kt);
                    if (r_win) {
#pragma unroll
                        for (int kt = 0; kt < 4; ++kt) {
                            const int4 kp = *reinterpret_cast<const int4*>(s_kpos + 16 * kt + 4 * G);
                            const int kpv[4] = {kp.x, kp.y, kp.z, kp.w};
#pragma unroll
                            for (int r = 0; r < 4; ++r)
                                if (!(kpv[r] > pos[t] - a.w && kpv[r] <= pos[t])) vm[t] &= ~(1u << (4 * kt + r));
                        }
                    }
                }
            }
        }
        uint32_t vm_any = vm[0];
#pragma unroll
        for (int t = 1; t < NRT; ++t) vm_any |= vm[t];
        if (__builtin_amdgcn_ballot_w64(vm_any != 0) != 0ull) {   // some row of this wave uses these keys
            // ---- S^T = K Q^T; every K fragment read from LDS serves all row tiles of the wave
            f32x4 s[NRT][4];
#pragma unroll
            for (int t = 0; t < NRT; ++t)
#pragma unroll
                for (int kt = 0; kt < 4; ++kt) s[t][kt] = f32x4{0.f, 0.f, 0.f, 0.f};
            auto k_frag = [&](int i) {   // fragment i: 16-key tile i % 4 of 64-byte chunk i / 4
                const int kc = i >> 2, kt = i & 3;
                return lds_read16(sK + ((kc & 1) ? k_rb_o : k_rb_e) + 16 * kt * KROWB + kc * 64);
            };
            if constexpr (BF16) {
                // issue order, pinned: 8 fragment reads ahead, then one read after each group of MFMAs, so that the
                // LDS latency of every fragment is covered by the MFMAs of the fragments before it
                constexpr int N_RD = 4 * KCH, LEAD = NRT == 1 ? 8 : 4;
                u32x4 kfb[LEAD];
#pragma unroll
                for (int i = 0; i < LEAD; ++i) kfb[i] = k_frag(i);
#pragma unroll
                for (int i = 0; i < N_RD; ++i) {
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int t = 0; t < NRT; ++t) s[t][i & 3] = mma_frag<BF16>(kfb[i % LEAD], qf[t][i >> 2], s[t][i & 3]);
                    if (i + LEAD < N_RD) kfb[i % LEAD] = k_frag(i + LEAD);
                }
            } else {
#pragma unroll
                for (int i = 0; i < 4 * KCH; ++i) {
                    const u32x4 kf = k_frag(i);
#pragma unroll
                    for (int t = 0; t < NRT; ++t) s[t][i & 3] = mma_frag<BF16>(kf, qf[t][i >> 2], s[t][i & 3]);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
            // ---- online softmax in the log2 domain (rows without a valid key keep their state: alpha = 1)
#pragma unroll
            for (int t = 0; t < NRT; ++t) {
                float mx = -INFINITY;
                // scores stay unscaled: the running maximum is kept in raw units and the scale (times log2 e)
                // is applied inside the exponent, one fused multiply-add per key
                if (__builtin_amdgcn_ballot_w64(vm[t] != 0xFFFFu) != 0ull) {   // uniform: some key is masked
#pragma unroll
                    for (int kt = 0; kt < 4; ++kt)
#pragma unroll
                        for (int r = 0; r < 4; ++r)
                            if (!((vm[t] >> (4 * kt + r)) & 1u)) s[t][kt][r] = -INFINITY;
                }
#pragma unroll
                for (int kt = 0; kt < 4; ++kt)
#pragma unroll
                    for (int r = 0; r < 4; ++r) mx = max_nan(mx, s[t][kt][r]);
                mx = xor16_max(mx);
                mx = xor32_max(mx);
                const float m_new = max_nan(mrun[t], mx);
                const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
                const float alpha = fast_exp2((mrun[t] - m_use) * a.scale_log2);
                const float neg_ms = -m_use * a.scale_log2;
                float rs = 0.f;
#pragma unroll
                for (int kt = 0; kt < 4; ++kt)
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const float pz = fast_exp2(__builtin_fmaf(s[t][kt][r], a.scale_log2, neg_ms));
                        s[t][kt][r] = pz;
                        rs += pz;
                    }
                rs = xor16_add(rs);
                rs = xor32_add(rs);
                zrun[t] = zrun[t] * alpha + rs;
                mrun[t] = m_new;
                if (__builtin_amdgcn_ballot_w64(alpha != 1.f) != 0ull) {      // uniform: some running max moved
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) acc[t][mt] *= alpha;
                }
            }
            __builtin_amdgcn_sched_barrier(0);
            // ---- O^T += V^T P^T; every V^T fragment read from LDS serves all row tiles of the wave
            if constexpr (BF16) {
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    u32x4 pb[NRT];
#pragma unroll
                    for (int t = 0; t < NRT; ++t) {
                        bf16x8 pk;
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            pk[r] = (__bf16)s[t][2 * u][r];
                            pk[4 + r] = (__bf16)s[t][2 * u + 1][r];
                        }
                        pb[t] = __builtin_bit_cast(u32x4, pk);
                    }
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) {
                        // keys 32 u + 4 G + e and 32 u + 16 + 4 G + e (e = 0..3) of column 16 mt + n: the order of pb
                        const u32x2 v0 = lds_read_tr16(sVT + vt_rb + (32 * u) * VR + mt * 32);
                        const u32x2 v1 = lds_read_tr16(sVT + vt_rb + (32 * u + 16) * VR + mt * 32);
                        const u32x4 vf = {v0[0], v0[1], v1[0], v1[1]};
#pragma unroll
                        for (int t = 0; t < NRT; ++t) acc[t][mt] = mma_frag<true>(vf, pb[t], acc[t][mt]);
                    }
                    {
                        constexpr int LEAD = 4;      // fragments (two reads each) ahead of their MFMAs
                        __builtin_amdgcn_sched_group_barrier(0x100, 2 * LEAD, 0);
#pragma unroll
                        for (int i = 0; i < MT - LEAD; ++i) {
                            __builtin_amdgcn_sched_group_barrier(0x008, NRT, 0);
                            __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
                        }
                        __builtin_amdgcn_sched_group_barrier(0x008, LEAD * NRT, 0);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            } else {
#pragma unroll
                for (int kt = 0; kt < 4; ++kt) {
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) {
                        const u32x4 vf = lds_read16(sVT + (16 * mt + n) * VP + (16 * kt + 4 * G) * 4);
#pragma unroll
                        for (int t = 0; t < NRT; ++t)
                            acc[t][mt] = mma_frag<false>(vf, __builtin_bit_cast(u32x4, s[t][kt]), acc[t][mt]);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
    };
    // One segment; joint slicing: the part's window tiles, then its schedule entries, a state for each.
    int out_slot = slot;
    for (int seg = 0; seg < (joint ? 2 : 1); ++seg) {
        if (joint) {
            r_win = seg == 0;
            r_slc = seg == 1;
            t0 = seg == 0 ? jw0 : js0;
            t1 = seg == 0 ? jw1 : js1;
            out_slot = a.n_cmp_chunks + seg * a.joint + part;
            if (seg) __syncthreads();     // every wave has finished reading the window's last tile
        }
#pragma unroll
        for (int t = 0; t < NRT; ++t) {
            mrun[t] = -INFINITY;
            zrun[t] = 0.f;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) acc[t][mt] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
        for (int j = 0; j < AHEAD; ++j)
            if (t0 + j < t1) issue_tile(t0 + j, vregs[j]);
        for (int it = t0; it < t1; it += AHEAD) {
#pragma unroll
            for (int j = 0; j < AHEAD; ++j)
                if (it + j < t1) tile_step(it + j, vregs[j]);
        }

        // ---- partial state of this slice: (m, Z) per row and the un-normalised accumulator
#pragma unroll
        for (int t = 0; t < NRT; ++t) {
            if (!rvalid[t]) continue;
            const int64_t pr = (int64_t)out_slot * a.rows_total + grow[t];
            if (G == 0) {
                a.part_stats[pr * 2 + 0] = mrun[t] * a.scale_log2;   // statistics leave the kernel in the log2 domain
                a.part_stats[pr * 2 + 1] = zrun[t];
                // work table: the sequence's last slice marks the compressed slots beyond its slices as empty
                if (r_cmp && cmp_parts && part == cmp_parts - 1) {
                    for (int sl = cmp_parts; sl < a.n_cmp_chunks; ++sl)
                        *reinterpret_cast<float2*>(a.part_stats + ((int64_t)sl * a.rows_total + grow[t]) * 2) = make_float2(0.f, 0.f);
                }
            }
            if (zrun[t] > 0.f) {
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
                    *reinterpret_cast<f32x4*>(a.part_acc + pr * DV + 16 * mt + 4 * G) = acc[t][mt];
            }
        }
    }
}

}  // namespace ssv
