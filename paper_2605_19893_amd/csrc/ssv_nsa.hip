// Host side of the C ABI declared in include/ssv_nsa.h: argument validation, launch planning,
// and the launch sequences of the refresh (Section 5.1) and reuse (Section 5.2) paths.
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <atomic>
#include <cmath>
#include <cstring>

#include "../../include/ssv_nsa.h"
#include "k_combine.hpp"
#include "k_compress.hpp"
#include "k_importance.hpp"
#include "k_scan32.hpp"
#include "k_stream.hpp"
#include "k_topn.hpp"
#include "planner.hpp"
#include "work_table.hpp"

// Scratch of ssv_nsa_verify_static: one copy per GPU inside the library's device image.  In host code this name is
// only a handle for hipGetSymbolAddress; the device address it resolves to is what kernels and copies are given.
static __device__ __align__(256) unsigned char scratch[SSV_STATIC_SCRATCH_BYTES];

namespace {

using namespace ssv;

struct Shape { int dtype, d_k, d_v; };
constexpr int kMaxDevices = 64;   // per-device one-time set-up flags
constexpr Shape kShapes[] = {{SSV_BF16, 192, 128}, {SSV_BF16, 128, 128}, {SSV_BF16, 64, 64}, {SSV_F32, 64, 64}};

int ceil_div(int a, int b) { return (a + b - 1) / b; }
size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Planning constants (measured choices; none is read from the environment).
constexpr int kResidentWgs = 256 * 2;        // workgroups one round holds: LDS and registers allow two per CU
constexpr int kMinTilesPerSlice = 2;
constexpr int kMinTilesMultiRound = 4;       // launches of several rounds: slices of a short sequence hold at least this many tiles
constexpr int kLongSliceTiles = 32;          // slice length once a launch needs several rounds (max_slice_tiles = 0)
constexpr int kImportanceWgs = 512;          // one round of the importance pass (more, shorter workgroups measured slower)
constexpr int kTopnInSlcMaxWgs = 256;        // SSV_TOPN_AUTO: select inside the selected-branch launch up to this many workgroups
                                             // (twice as many when a wavefront has one query to select for)
constexpr size_t kMaxStreamLds = 80 * 1024;  // two workgroups per CU
constexpr int kScan32Wgs = 256;              // the matrix-core scan: one workgroup per CU
constexpr int kScan32MinRows = 192;          // SSV_SCAN_AUTO: rows per (sequence, KV head) from which it is used ...
constexpr int kScan32MinTileSteps = 1024;    // ... when the launch has at least this many tile steps (four per CU)
constexpr int kTableMinTileSteps = 4096;     // the streaming scan of a mixed-length batch: tile steps from which a work table pays for its launch
constexpr int kScan32PairCost = 4;           // its balanced split: what a segment costs a workgroup besides its tiles, in tiles
constexpr int kScan32MinTilesMultiRound = 8; // its launches of several rounds: slices of a short sequence hold at least this many tiles
constexpr size_t kMaxLds = 160 * 1024;
constexpr int kCombineStreamWgs = 1024;       // resident workgroups of the streaming combine (four per CU)

struct Layout {
    ssv_nsa_plan plan;
    int H_g, es;
    bool one_launch, unfused, scan32;
    bool scan_balanced;          // matrix-core scan: equal ranges over the batch's tiles instead of even slices per group
    int scan_ranges, scan_range_min;
    int cmp_items_max;           // > 0: the streaming kernel's compressed scan takes its slices from a work table (k_work_table)
    bool table_kernel;           // the call starts with k_work_table
    int joint_parts;             // > 0: the <WIN|SLC> launch cuts window tiles and schedule entries of a group together
    int imp_items_max;           // > 0: the importance pass takes its slices from the work table the balanced scan writes
    int imp_C, imp_n_qg, n_imp_chunks, imp_rw;   // importance pass: routed queries per workgroup, such workgroups per sequence, slices, blocks of 64 rows per workgroup
    int nc_pitch, max_blocks, bitmap_words, max_sched;
    size_t lds_stream, lds_k, lds_vt;
    int64_t rows_total;
    int64_t q_s[3], out_s[3];            // bytes
    size_t off_stats, off_acc, off_colsum, off_branch, off_imp_table, off_cmp_table, branch_bytes, total;
};

// LDS tile sizes of the streaming kernel for a shape (they equal StreamCfg<...>::LDS_K / LDS_VT)
void stream_tile_lds(bool bf16, int d_k, int d_v, size_t* lds_k, size_t* lds_vt) {
    const int es = bf16 ? 2 : 4;
    *lds_k = (size_t)2 * kTile * d_k * es;
    *lds_vt = bf16 ? (size_t)kTile * (d_v * 2 + 32) : (size_t)d_v * (kTile * 4 + 16);
}

int make_layout(const ssv_nsa_params* p, Layout* lo) {
    if (!p) return SSV_EINVAL;
    if (p->B < 1 || p->T < 1 || p->H < 1 || p->H_kv < 1 || p->d_k < 1 || p->d_v < 1) return SSV_EINVAL;
    if (p->H % p->H_kv) return SSV_EINVAL;
    if (p->l < 1 || p->d < 1 || p->l % p->d || p->l_sel < 1 || p->l_sel % p->d) return SSV_EINVAL;
    if (p->n_sel < 1 || p->n_init < 0 || p->n_local < 0 || p->n_sel < p->n_init + p->n_local) return SSV_EINVAL;
    if (p->w < 1 || p->max_seq_len < 0 || p->max_n_cmp < 0 || p->avg_seq_len < 0 || p->avg_seq_len > p->max_seq_len) return SSV_EINVAL;
    if (p->dtype != SSV_F32 && p->dtype != SSV_BF16) return SSV_EINVAL;
    if (p->mode != SSV_REFRESH && p->mode != SSV_REUSE && p->mode != SSV_REFRESH_SHARED) return SSV_EINVAL;
    if (p->group_size < 0 || !(p->scale >= 0.f) || std::isinf(p->scale)) return SSV_EINVAL;
    if (p->exec != SSV_EXEC_FUSED && p->exec != SSV_EXEC_UNFUSED) return SSV_EINVAL;
    if (p->topn_home != SSV_TOPN_AUTO && p->topn_home != SSV_TOPN_SEPARATE && p->topn_home != SSV_TOPN_IN_SLC) return SSV_EINVAL;
    if (p->max_slice_tiles != 0 && (p->max_slice_tiles < 2 || p->max_slice_tiles > 64)) return SSV_EINVAL;
    if (p->imp_rows != 0 && p->imp_rows != 64 && p->imp_rows != 128 && p->imp_rows != 256) return SSV_EINVAL;
    if (p->scan_kernel < SSV_SCAN_AUTO || p->scan_kernel > SSV_SCAN_STREAM_TABLE) return SSV_EINVAL;
    const bool unfused = p->exec == SSV_EXEC_UNFUSED;
    if (p->scan_kernel == SSV_SCAN_MATRIX && (unfused || p->dtype != SSV_BF16)) return SSV_EINVAL;
    if (p->scan_kernel == SSV_SCAN_STREAM_TABLE && unfused) return SSV_EINVAL;
    if (unfused && (p->mode == SSV_REFRESH_SHARED || p->group_size > 1 || p->scan_group_size > 1)) return SSV_EINVAL;
    const int H_g = p->H / p->H_kv;
    if (p->T > SSV_MAX_T) return SSV_EUNSUPPORTED;
    if (H_g != 1 && H_g != 2 && H_g != 4 && H_g != 8 && H_g != 16) return SSV_EUNSUPPORTED;
    if (p->l_sel != kTile || p->n_sel > kMaxNSel) return SSV_EUNSUPPORTED;
    if (!ssv_nsa_supported(p->dtype, p->d_k, p->d_v)) return SSV_EUNSUPPORTED;
    const int es = p->dtype == SSV_BF16 ? 2 : 4;
    const int64_t* strides[4] = {p->k_stride, p->v_stride, p->kc_stride, p->vc_stride};
    const int dims[4] = {p->d_k, p->d_v, p->d_k, p->d_v};
    for (int a = 0; a < 4; ++a)
        for (int j = 0; j < 3; ++j) {
            if (strides[a][j] < 0 || (strides[a][j] * es) % 16) return SSV_EINVAL;
            if (j == 2 && strides[a][j] < dims[a]) return SSV_EINVAL;
        }
    // K rows are fetched through 32-bit buffer offsets from the start of a (sequence, KV head)
    if ((int64_t)(p->max_seq_len + p->T) * p->k_stride[2] * es >= (1ll << 31) ||
        (int64_t)p->max_n_cmp * p->kc_stride[2] * es >= (1ll << 31))
        return SSV_EUNSUPPORTED;
    const bool shared = p->mode == SSV_REFRESH_SHARED;
    const int c_max = shared ? p->T : std::min(p->T, std::min(64, 128 / H_g));   // ownership masks hold 64 queries
    if (p->group_size > c_max) return SSV_EINVAL;
    const bool force32 = p->scan_kernel == SSV_SCAN_MATRIX;
    if (p->scan_group_size < 0 || p->scan_group_size > std::min(p->T, force32 ? 256 / H_g : std::min(64, 128 / H_g))) return SSV_EINVAL;
    // (the matrix-core scan fetches V rows through 32-bit buffer offsets as well)
    if (force32 && (int64_t)p->max_n_cmp * p->vc_stride[2] * es >= (1ll << 31)) return SSV_EUNSUPPORTED;
    const int max_blocks = (p->max_seq_len + p->T) / p->l_sel + 1;
    if (max_blocks > 16384) return SSV_EUNSUPPORTED;

    std::memset(lo, 0, sizeof(*lo));
    lo->unfused = unfused;
    // q and out: all-zero strides mean contiguous [B, T, H, d]
    {
        const int64_t* given[2] = {p->q_stride, p->out_stride};
        int64_t* bytes[2] = {lo->q_s, lo->out_s};
        const int dd[2] = {p->d_k, p->d_v};
        for (int a = 0; a < 2; ++a) {
            const bool dense = !given[a][0] && !given[a][1] && !given[a][2];
            const int64_t st[3] = {dense ? (int64_t)p->T * p->H * dd[a] : given[a][0], dense ? (int64_t)p->H * dd[a] : given[a][1],
                                   dense ? (int64_t)dd[a] : given[a][2]};
            for (int j = 0; j < 3; ++j) {
                if (st[j] < 0 || (st[j] * es) % 16) return SSV_EINVAL;
                bytes[a][j] = st[j] * es;
            }
            if (st[2] < dd[a] || st[1] < dd[a] || (p->B > 1 && st[0] < dd[a])) return SSV_EINVAL;
        }
    }
    ssv_nsa_plan& pl = lo->plan;
    // default: 64 rows per workgroup (one 16-row tile per wave keeps the software pipeline in registers);
    // up to 128 rows (two row tiles per wave) on request
    // (the shared-index variant keeps this automatic grouping: its group_size is the sharing group)
    pl.C = unfused ? 1 : ((p->group_size && !shared) ? p->group_size : std::max(1, std::min(p->T, 64 / H_g)));
    pl.share_group = shared ? (p->group_size ? p->group_size : pl.C) : 0;
    pl.n_qg = ceil_div(p->T, pl.C);
    pl.rows_per_wg = pl.C * H_g;
    // Split plan.  A launch should fill the chip once with resident workgroups (LDS and registers allow two per
    // CU), so the key tiles of a (sequence, head, query group) are cut into about capacity / units slices, but
    // never below min_tiles tiles per slice.  Small problems take one workgroup per CU instead (a workgroup that
    // has its CU to itself runs a tile in 2.3 us instead of 3.3): when that leaves slices of at most four tiles.
    const int units = p->B * p->H_kv * pl.n_qg;
    const int capacity = kResidentWgs;
    const int ntc = std::max(1, ceil_div(p->max_n_cmp, kTile));         // compressed tiles of the longest sequence
    // an average sequence has fewer compressed tiles than the longest one: budget slices for the average, so
    // that slices of long and short sequences come out at about the same length
    const double avg_frac = (p->avg_seq_len > 0 && p->max_seq_len > 0) ? (double)p->avg_seq_len / p->max_seq_len : 1.0;
    const int ntc_avg = std::max(1, (int)std::ceil(ntc * avg_frac));
    const int ntw = (p->w + p->T) / kTile + 2;                          // window tiles
    // Scan grouping.  The compressed and window scans read the same rows for every query of a sequence, so when the
    // chip is kept busy for several rounds by them (8 tile steps or more per resident workgroup) their launch takes
    // groups of up to 128 rows (two row tiles per wave share every K and V fragment read from LDS: measured 18-20 %
    // faster at 16-40 queries per sequence), balanced over the sequence's queries.  An explicit group_size applies
    // to both launches unless the scan has one of its own.
    // The matrix-core scan (bf16): groups of up to 256 rows, one workgroup per CU.  Automatic where a KV head has
    // enough rows to fill most of such a workgroup and the launch runs for several tiles per CU: there the scan is
    // bound by the matrix cores, and the streaming kernel's 128-row workgroups re-read every tile from L2.
    {
        const int n_g32 = ceil_div(p->T * H_g, 256);
        const bool can32 = !unfused && p->dtype == SSV_BF16 && (int64_t)p->max_n_cmp * p->vc_stride[2] * es < (1ll << 31);
        lo->scan32 = force32 || (p->scan_kernel == SSV_SCAN_AUTO && can32 && !p->scan_group_size && (!p->group_size || shared) &&
                                 p->T * H_g >= kScan32MinRows &&
                                 (int64_t)p->B * p->H_kv * n_g32 * ntc_avg >= kScan32MinTileSteps);
    }
    pl.C_scan = pl.C;
    if (unfused) pl.C_scan = 1;
    else if (lo->scan32) {
        const int c_cap = std::max(1, std::min(p->T, 256 / H_g));
        pl.C_scan = p->scan_group_size ? p->scan_group_size : ceil_div(p->T, ceil_div(p->T, c_cap));   // balanced over the groups
    }
    else if (p->scan_group_size) pl.C_scan = p->scan_group_size;
    else if (!p->group_size || shared) {
        const int n_a = ceil_div(p->T, std::max(1, std::min(p->T, 128 / H_g)));
        const int cand = ceil_div(p->T, n_a);
        if (cand > pl.C && (int64_t)units * (ntc_avg + ntw) >= 8 * (int64_t)capacity) pl.C_scan = cand;
    }
    pl.n_qg_scan = ceil_div(p->T, pl.C_scan);
    const int units_scan = p->B * p->H_kv * pl.n_qg_scan;
    pl.max_sched_entries = pl.C * p->n_sel;
    // selected tiles, at most; with one shared index set per group the schedule is a single set
    const int nts = shared ? ceil_div(pl.C, pl.share_group) * p->n_sel : pl.max_sched_entries;
    pl.min_tiles_per_split = kMinTilesPerSlice;
    const int mt = pl.min_tiles_per_split;
    const int long_slice = p->max_slice_tiles ? p->max_slice_tiles : kLongSliceTiles;
    // Tiles per slice.  If one round of resident workgroups can take the launch with slices of at most long_slice
    // tiles, `per` is grown until the slices of an average unit fit the capacity (no partial second round).
    // Otherwise slices are cut to long_slice tiles: several rounds of workgroups, and the longest slice, the long
    // pole of a mixed-length batch, stays bounded (12-tile slices balanced better but cost 5-10 % at the
    // 128K-context configurations: twice the partial states to write and merge, twice the per-workgroup start-up).
    auto tiles_per_slice = [&](const int* tiles, int n_roles, int n_units) {
        int total = 0;
        for (int r = 0; r < n_roles; ++r) total += tiles[r];
        int spu = std::max(n_roles, (capacity / 2) / n_units);      // slices per unit one round can hold, one workgroup per CU
        if (std::max(mt, ceil_div(total, spu)) > 4) spu = std::max(n_roles, capacity / n_units);   // two per CU
        int per = std::max(mt, ceil_div(total, spu));
        if (per > long_slice) return long_slice;
        for (;; ++per) {
            int sum = 0;
            for (int r = 0; r < n_roles; ++r) sum += std::max(1, ceil_div(tiles[r], per));
            if (sum <= spu || per >= total) return per;
        }
    };
    int per_c, per_w, per_s;
    lo->one_launch = !unfused && !lo->scan32 && p->mode == SSV_REUSE && pl.C_scan == pl.C;   // all three branches in one launch
    if (unfused) {              // one launch per branch
        per_c = tiles_per_slice(&ntc_avg, 1, units);
        per_w = tiles_per_slice(&ntw, 1, units);
        per_s = tiles_per_slice(&nts, 1, units);
    } else if (lo->scan32) {
        // the scan: slices so that the average unit fills one round of one workgroup per CU, cut to long_slice tiles
        // when that takes several rounds; window and selected blocks share the second launch
        const int spu = std::max(1, kScan32Wgs / units_scan);
        per_c = std::min(std::max(1, ceil_div(ntc_avg, spu)), long_slice);
        const int tiles_b = ntw + nts;      // (cut as one list: a part may end the window and begin the schedule)
        per_w = per_s = tiles_per_slice(&tiles_b, 1, units);
    } else if (lo->one_launch) {
        const int tiles[3] = {ntc_avg, ntw, nts};
        per_c = per_w = per_s = tiles_per_slice(tiles, 3, units);
    } else {
        const int tiles_a[2] = {ntc_avg, ntw};
        per_c = per_w = tiles_per_slice(tiles_a, 2, units_scan);
        per_s = tiles_per_slice(&nts, 1, units);
    }
    // (caps: the combine kernel's per-row slice loops; unfused: every branch is merged by thread groups that own rows)
    const int cap_c = unfused ? kCombineRowsMaxSlots : kMaxSlotsPerBranch, cap_ws = unfused ? kCombineRowsMaxSlots : 32;
    pl.n_cmp_chunks = std::min(std::max(1, ceil_div(ntc, per_c)), cap_c);
    // The matrix-core scan of a batch of mixed lengths (the caller's average is below the maximum): one range of the
    // batch's tile sequence per workgroup, about total / 256 tiles each; the lengths are read on the device, the
    // average only sizes the slots: a pair of the longest sequence is cut by at most ceil(ntc / range) + 1 ranges, and
    // the kernel never takes ranges shorter than scan_range_min (in tiles plus the fixed cost per pair), which keeps every
    // pair within the slots there are.
    lo->scan_balanced = false;
    lo->scan_ranges = lo->scan_range_min = 0;
    if (lo->scan32 && ntc_avg < ntc && p->B <= kScan32MaxBalancedB && (int64_t)p->B * p->H_kv * (ntc + kScan32PairCost) < (1ll << 30)) {
        lo->scan_balanced = true;
        lo->scan_ranges = std::max(1, kScan32Wgs / pl.n_qg_scan);
        const int cost = ntc + kScan32PairCost;                      // of a pair of the longest sequence
        const int range_est = std::max(1, ceil_div(p->B * p->H_kv * (ntc_avg + kScan32PairCost), lo->scan_ranges));
        pl.n_cmp_chunks = std::min(std::max(2, ceil_div(cost, range_est) + 1), cap_c);
        lo->scan_range_min = ceil_div(cost, pl.n_cmp_chunks - 1);
        per_c = std::max(range_est, lo->scan_range_min);
    }
    pl.n_win_splits = std::min(std::max(1, ceil_div(ntw, per_w)), cap_ws);
    pl.n_slc_splits = std::min(std::max(1, ceil_div(nts, per_s)), cap_ws);
    lo->joint_parts = 0;
    if (lo->scan32) {
        // One round of resident workgroups: the parts of a group are cut over window tiles and schedule entries together,
        // and every part owns a window slot and a selected slot (the one its tiles do not reach stays empty); measured
        // 3 us faster at a 40-node tree over 128K tokens, where the window's own workgroup would sit idle for half the
        // launch.  Several rounds fill such gaps by themselves (32 mixed-length sequences: 2 us slower): separate slices.
        const int parts = std::min(std::max(1, ceil_div(ntw + nts, per_s)), kCombineRowsMaxSlots / 2);
        if (units * parts <= kResidentWgs) {
            lo->joint_parts = parts;
            pl.n_win_splits = pl.n_slc_splits = parts;
        } else {
            const int tiles_b[2] = {ntw, nts};
            per_w = per_s = tiles_per_slice(tiles_b, 2, units);
            pl.n_win_splits = std::min(std::max(1, ceil_div(ntw, per_w)), cap_ws);
            pl.n_slc_splits = std::min(std::max(1, ceil_div(nts, per_s)), cap_ws);
        }
    }
    // The streaming kernel's compressed scan of a batch of mixed lengths: slices per sequence in proportion to its length,
    // from a work table that a one-workgroup kernel builds from the device-resident lengths at the start of the call
    // (work_table.hpp).  One round: the resident workgroups that the launch's other branches leave, at least two items
    // per sequence; the slots per row bound the slices of the longest sequence (sized from the average, enforced by the
    // table).  Only where the scan is long enough for the extra launch (5 to 7 us) to pay.
    lo->cmp_items_max = 0;
    const bool force_table = p->scan_kernel == SSV_SCAN_STREAM_TABLE;
    if (!unfused && !lo->scan32 && p->B <= kWorkTableMaxB &&
        (force_table || (ntc_avg < ntc && (int64_t)units_scan * ntc_avg >= kTableMinTileSteps))) {
        const int others = units_scan * (pl.n_win_splits + (lo->one_launch ? pl.n_slc_splits : 0));
        const int items = (kResidentWgs - others) / (p->H_kv * pl.n_qg_scan);
        if (items >= 2 * p->B) {
            lo->cmp_items_max = items;
            const int64_t total_est = (int64_t)p->B * ntc_avg;
            pl.n_cmp_chunks = (int)std::min<int64_t>(cap_c, std::max<int64_t>(1, ((int64_t)ntc * (items - p->B) + total_est - 1) / total_est + 1));
            per_c = ceil_div(ntc, pl.n_cmp_chunks);
        }
    }
    pl.tiles_per_chunk = lo->scan_balanced ? per_c : ceil_div(ntc, pl.n_cmp_chunks);
    pl.n_slots = pl.n_cmp_chunks + pl.n_win_splits + pl.n_slc_splits;

    lo->H_g = H_g;
    // importance pass: every query is routed, or one representative per group of C (shared-index variant), then
    // packed 64, 128 or 256 rows to a workgroup; 2 workgroups per CU are resident (72 KB of LDS each for the K strips
    // in flight): one round of at most 512 (more, shorter workgroups measured slower: every workgroup pays about
    // 10 us of start-up before its first tile).  With 64 rows per workgroup every workgroup streams its whole slice
    // of k_cmp from L2 for those 64 rows, which is what bounds the pass once a KV head has several hundred rows;
    // wider workgroups share every strip between 2 or 4 row blocks.  Small problems keep 64 rows: more workgroups,
    // each with one or two tiles.
    const int routed = shared ? ceil_div(p->T, pl.share_group) : p->T;
    const int rows_routed = routed * H_g;
    // (an explicit group_size, like the unfused execution, also sets the queries per workgroup of this pass, so that
    // per-query execution is per-query throughout)
    const bool own_groups = !shared && (p->group_size || unfused);
    int rw = 1;
    if (p->imp_rows) rw = p->imp_rows / 64;
    else if (!own_groups) {
        // wide only where the wide workgroups still get four tiles or more each
        for (int cand = rows_routed >= 256 ? 4 : (rows_routed >= 128 ? 2 : 1); cand > 1 && rw == 1; cand /= 2)
            if ((int64_t)p->B * p->H_kv * ceil_div(rows_routed, 64 * cand) * ntc_avg >= 4 * (int64_t)kImportanceWgs) rw = cand;
    }
    while (rw > 1 && rows_routed <= 64 * (rw / 2)) rw /= 2;         // no more row blocks than the rows fill
    lo->imp_rw = rw;
    {
        int c_cap = std::max(1, 64 * rw / H_g);                         // queries one workgroup can hold
        if (own_groups && !p->imp_rows) c_cap = std::min(c_cap, pl.C);
        const int n_g = ceil_div(routed, c_cap);
        lo->imp_C = ceil_div(routed, n_g);                              // balanced over the groups
        lo->imp_n_qg = ceil_div(routed, lo->imp_C);
    }
    const int imp_units = p->B * p->H_kv * lo->imp_n_qg;
    lo->n_imp_chunks = std::max(1, std::min(ntc, std::max(1, kImportanceWgs / imp_units)));
    // a refresh call of a mixed-length batch: slices per sequence in proportion to its length, from the work table that
    // the balanced scan or the table kernel writes (one round of about equally long workgroups; needs room for two
    // items per sequence at least; the 32x32x16 kernel only)
    lo->imp_items_max = 0;
    if ((lo->scan_balanced || (lo->cmp_items_max && p->dtype == SSV_BF16)) && p->mode != SSV_REUSE) {
        const int items = kImportanceWgs / (p->H_kv * lo->imp_n_qg);
        if (items >= 2 * p->B) lo->imp_items_max = items;
    }
    lo->table_kernel = lo->cmp_items_max > 0;      // (it builds the importance pass's table too)
    lo->es = es;
    lo->nc_pitch = (int)align_up((size_t)std::max(1, p->max_n_cmp), kTile);
    lo->max_blocks = max_blocks;
    // rounded so that every LDS array behind them stays 16-byte aligned
    lo->bitmap_words = (ceil_div(max_blocks, 32) + 1) & ~1;
    lo->max_sched = (pl.max_sched_entries + 3) & ~3;
    stream_tile_lds(p->dtype == SSV_BF16, p->d_k, p->d_v, &lo->lds_k, &lo->lds_vt);
    lo->lds_stream = stream_lds_bytes(lo->lds_k, lo->lds_vt, lo->max_sched, lo->bitmap_words);
    if (lo->lds_stream > kMaxStreamLds) return SSV_EUNSUPPORTED;     // merged schedules of very large groups do not fit
    // Top-n selection of a refresh call: inside the selected-branch launch (every workgroup selects for its own
    // group's queries, one query per wavefront, in the tile buffers that are idle until the schedule exists) when the
    // importance arrays of four queries fit there.  Every slice of a group repeats the group's selections, which
    // costs nothing while the launch leaves CUs idle (at most one workgroup per CU) and is slower than the
    // separate launch once the chip is full.
    const bool refresh = p->mode != SSV_REUSE;
    const bool fits = fused_topn_lds_bytes(max_blocks, pl.C, p->n_sel) <= lo->lds_k + lo->lds_vt;
    const int n_wg_b = units * (lo->joint_parts ? lo->joint_parts : pl.n_slc_splits + (lo->scan32 ? pl.n_win_splits : 0));
    pl.topn_in_slc = refresh && !unfused && fits &&
                     (p->topn_home == SSV_TOPN_IN_SLC || (p->topn_home == SSV_TOPN_AUTO && n_wg_b <= (pl.C <= 4 ? 2 : 1) * kTopnInSlcMaxWgs));
    pl.n_imp_chunks = refresh ? lo->n_imp_chunks : 0;
    pl.imp_rows = refresh ? 64 * lo->imp_rw : 0;
    if (unfused) pl.n_launches = refresh ? 9 : 7;
    else pl.n_launches = (lo->one_launch ? 1 : 2) + (refresh ? 1 + !pl.topn_in_slc : 0) + 1 + (lo->table_kernel ? 1 : 0);
    pl.scan_matrix = lo->scan32;
    lo->rows_total = (int64_t)p->B * p->T * p->H;
    size_t off = 0;
    lo->off_stats = off;
    off = align_up(off + (size_t)pl.n_slots * lo->rows_total * 2 * sizeof(float), 256);
    lo->off_acc = off;
    off = align_up(off + (size_t)pl.n_slots * lo->rows_total * p->d_v * sizeof(float), 256);
    lo->off_colsum = off;
    off = align_up(off + (size_t)p->B * p->T * p->H_kv * lo->nc_pitch * sizeof(float), 256);
    lo->off_branch = off;
    lo->branch_bytes = align_up((size_t)lo->rows_total * p->d_v * es, 256);
    if (unfused) off += 3 * lo->branch_bytes;    // the three branch outputs, [rows, d_v] in the storage type
    lo->off_imp_table = off;
    if (lo->imp_items_max) off = align_up(off + work_table_bytes(lo->imp_items_max), 256);
    lo->off_cmp_table = off;
    if (lo->cmp_items_max) off = align_up(off + work_table_bytes(lo->cmp_items_max), 256);
    lo->total = off;
    pl.workspace_bytes = (int64_t)off;
    return SSV_OK;
}

// The importance kernel of a shape: bf16 on the 32x32x16 matrix instruction, fp32 on 16x16x4; by heads-per-group class
// (16, 4, 1) and blocks of 64 rows per workgroup (1, 2, 4).
template <bool BF16, int DK>
struct ImportanceKernels {
    static constexpr size_t LDS = BF16 ? (size_t)Importance32Cfg<DK>::LDS_RING : (size_t)ImportanceCfg<false, DK>::LDS_RING;
    // wavefronts per workgroup: the 256-row bf16 kernel of 16-head groups runs with eight (the other head classes need
    // more than the 128 registers that four wavefronts per SIMD leave each)
    static constexpr int waves(int hgm, int rw) { return (BF16 && hgm == 16 && rw == 4) ? 8 : 4; }
    template <int HGM, int RW>
    static const void* one() {
        if constexpr (BF16) return (const void*)k_importance32<DK, HGM, RW, waves(HGM, RW)>;
        else return (const void*)k_importance<false, DK, HGM, RW>;
    }
    static const void* fn(int hgm, int rw) {
#define SSV_IMP_ROW(HGM_) (rw == 4 ? one<HGM_, 4>() : (rw == 2 ? one<HGM_, 2>() : one<HGM_, 1>()))
        return hgm == 16 ? SSV_IMP_ROW(16) : (hgm == 4 ? SSV_IMP_ROW(4) : SSV_IMP_ROW(1));
#undef SSV_IMP_ROW
    }
};

struct Timer {
    bool on = false;
    int repeats = 1;     // timed mode: every kernel is launched this many times back to back (all are idempotent)
    hipStream_t stream = nullptr;
    hipEvent_t ev[SSV_NUM_TIMINGS][2] = {};
    bool used[SSV_NUM_TIMINGS] = {};
    // One launch per kernel: its start and stop events are bound to the launch itself and read the dispatch's own
    // begin and end, which is the duration a kernel trace reports.  Several launches: one event pair around them.
    bool per_dispatch() const { return on && repeats == 1; }
    int begin(int k, bool bracket_only = false) {
        if (!on) return 0;
        if (hipEventCreate(&ev[k][0]) != hipSuccess || hipEventCreate(&ev[k][1]) != hipSuccess) return -1;
        used[k] = true;
        if (per_dispatch() && !bracket_only) return 0;
        return hipEventRecord(ev[k][0], stream) == hipSuccess ? 0 : -1;
    }
    int end(int k, bool bracket_only = false) {
        if (!on || (per_dispatch() && !bracket_only)) return 0;
        return hipEventRecord(ev[k][1], stream) == hipSuccess ? 0 : -1;
    }
    int finish(float* ms) {
        int rc = 0;
        if (!on) return 0;
        if (hipStreamSynchronize(stream) != hipSuccess) rc = -1;
        for (int k = 0; k < SSV_NUM_TIMINGS; ++k) {
            ms[k] = 0.f;
            if (used[k]) {
                if (rc == 0 && hipEventElapsedTime(&ms[k], ev[k][0], ev[k][1]) != hipSuccess) rc = -1;
                if (k < SSV_NUM_KERNELS) ms[k] /= (float)repeats;
                (void)hipEventDestroy(ev[k][0]);
                (void)hipEventDestroy(ev[k][1]);
            }
        }
        return rc;
    }
};

// Launch of timed kernel K_: with its own start/stop events when every kernel is launched once, plainly otherwise.
#define SSV_LAUNCH_T(K_, KERNEL_, GRID_, THREADS_, LDS_, ARGS_)                                                          \
    do {                                                                                                                 \
        if (tm.per_dispatch())                                                                                           \
            hipExtLaunchKernelGGL(KERNEL_, dim3(GRID_), dim3(THREADS_), (uint32_t)(LDS_), stream, tm.ev[K_][0], tm.ev[K_][1], 0, ARGS_); \
        else                                                                                                             \
            hipLaunchKernelGGL(KERNEL_, dim3(GRID_), dim3(THREADS_), LDS_, stream, ARGS_);                               \
    } while (0)
#define SSV_LAUNCH(K_, KERNEL_, GRID_, LDS_, ARGS_) SSV_LAUNCH_T(K_, KERNEL_, GRID_, kThreads, LDS_, ARGS_)

template <bool BF16, int DK, int DV>
int launch_all(const void* q, const void* k, const void* v, const void* kc, const void* vc, const float* gates,
               const int32_t* seq_lens, const int32_t* n_cmp, const int32_t* n_query, const int32_t* parents,
               const ssv_nsa_params* p, void* out, int32_t* sel_idx, char* ws, const Layout& lo, hipStream_t stream,
               Timer& tm) {
    using SC = StreamCfg<BF16, DK, DV>;
    static_assert(SC::LDS_K == 2 * kTile * DK * (BF16 ? 2 : 4), "stream_tile_lds must describe this shape");
    const ssv_nsa_plan& pl = lo.plan;
    const int es = lo.es;
    const float scale = p->scale > 0.f ? p->scale : 1.0f / std::sqrt((float)p->d_k);
    const float scale_log2 = scale * 1.4426950408889634f;
    float* part_stats = reinterpret_cast<float*>(ws + lo.off_stats);
    float* part_acc = reinterpret_cast<float*>(ws + lo.off_acc);
    float* colsum = reinterpret_cast<float*>(ws + lo.off_colsum);
    if ((size_t)SC::LDS_K != lo.lds_k || (size_t)SC::LDS_VT != lo.lds_vt) return SSV_EUNSUPPORTED;   // (cannot happen)

    StreamArgs sa{};
    sa.q = (const char*)q; sa.k = (const char*)k; sa.v = (const char*)v; sa.kc = (const char*)kc; sa.vc = (const char*)vc;
    sa.seq_lens = seq_lens; sa.n_cmp = n_cmp; sa.n_query = n_query; sa.parents = parents; sa.sel_idx = sel_idx;
    sa.part_stats = part_stats; sa.part_acc = part_acc;
    sa.B = p->B; sa.T = p->T; sa.H = p->H; sa.H_kv = p->H_kv; sa.H_g = lo.H_g; sa.C = pl.C; sa.n_qg = pl.n_qg;
    sa.l = p->l; sa.d = p->d; sa.n_sel = p->n_sel; sa.w = p->w; sa.scale_log2 = scale_log2;
    sa.max_seq_len = p->max_seq_len; sa.max_n_cmp = p->max_n_cmp;
    sa.n_cmp_chunks = pl.n_cmp_chunks; sa.n_win_splits = pl.n_win_splits; sa.n_slc_splits = pl.n_slc_splits;
    sa.min_tiles = 1;     // inside a launch the used slices share the tiles evenly, down to one tile each (launch_stream
                          // raises this for launches of several rounds)
    sa.max_sched = lo.max_sched; sa.bitmap_words = lo.bitmap_words; sa.rows_total = lo.rows_total;
    for (int j = 0; j < 3; ++j) {
        sa.k_s[j] = p->k_stride[j] * es; sa.v_s[j] = p->v_stride[j] * es;
        sa.kc_s[j] = p->kc_stride[j] * es; sa.vc_s[j] = p->vc_stride[j] * es;
        sa.q_s[j] = lo.q_s[j];
    }
    const size_t lds_stream = lo.lds_stream;
    {
        // kernels that may ask for more than 64 KB of dynamic LDS: raise their limit once per device (repeating the
        // calls after a lost race between two host threads is harmless)
        static std::atomic<bool> raised[kMaxDevices];
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return SSV_ELAUNCH;
        if (!raised[dev].load(std::memory_order_acquire)) {
            const void* fns[] = {(const void*)k_stream<BF16, DK, DV, 1, kRolesAll>, (const void*)k_stream<BF16, DK, DV, 1, kRolesSlc>,
                                 (const void*)k_stream<BF16, DK, DV, 1, kRolesCmpWin>, (const void*)k_stream<BF16, DK, DV, 2, kRolesAll>,
                                 (const void*)k_stream<BF16, DK, DV, 2, kRolesSlc>, (const void*)k_stream<BF16, DK, DV, 2, kRolesCmpWin>,
                                 (const void*)k_stream<BF16, DK, DV, 1, kRolesCmp>, (const void*)k_stream<BF16, DK, DV, 1, kRolesWin>,
                                 (const void*)k_stream<BF16, DK, DV, 1, kRolesWinSlc>, (const void*)k_stream<BF16, DK, DV, 2, kRolesWinSlc>,
                                 ImportanceKernels<BF16, DK>::fn(16, 1), ImportanceKernels<BF16, DK>::fn(4, 1), ImportanceKernels<BF16, DK>::fn(1, 1),
                                 ImportanceKernels<BF16, DK>::fn(16, 2), ImportanceKernels<BF16, DK>::fn(4, 2), ImportanceKernels<BF16, DK>::fn(1, 2),
                                 ImportanceKernels<BF16, DK>::fn(16, 4), ImportanceKernels<BF16, DK>::fn(4, 4), ImportanceKernels<BF16, DK>::fn(1, 4)};
            for (const void* fn : fns)
                if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kMaxStreamLds) != hipSuccess) return SSV_ELAUNCH;
            if constexpr (BF16) {
                if (hipFuncSetAttribute((const void*)k_scan32<DK, DV, false>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                        (int)Scan32Cfg<DK, DV>::LDS) != hipSuccess ||
                    hipFuncSetAttribute((const void*)k_scan32<DK, DV, true>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                        (int)Scan32Cfg<DK, DV>::LDS) != hipSuccess)
                    return SSV_ELAUNCH;
            }
            raised[dev].store(true, std::memory_order_release);
        }
    }

    const int reps = tm.on ? tm.repeats : 1;
    // one k_stream launch over the partial-state slots [slot_lo, slot_lo + slot_cnt) with query groups of C
    auto launch_stream = [&](int K, int roles, int slot_lo, int slot_cnt, int C, int n_qg) -> int {
        sa.C = C; sa.n_qg = n_qg;
        sa.slot_lo = slot_lo; sa.slot_cnt = slot_cnt; sa.n_wg = p->B * p->H_kv * n_qg * slot_cnt;
        // the compressed scan from its work table: its workgroups first, then those of the launch's other branches
        const bool tabled = lo.cmp_items_max > 0 && (roles & 1);
        sa.cmp_table = tabled ? reinterpret_cast<const int32_t*>(ws + lo.off_cmp_table) : nullptr;
        sa.cmp_items_max = lo.cmp_items_max;
        if (tabled) sa.n_wg = (lo.cmp_items_max + p->B * (slot_cnt - pl.n_cmp_chunks)) * p->H_kv * n_qg;
        // A launch of several rounds of workgroups gains nothing from cutting a short sequence into slices of one
        // or two tiles: every slice pays the start-up of a workgroup and leaves a partial state to merge.
        sa.min_tiles = sa.n_wg > kResidentWgs ? kMinTilesMultiRound : 1;
        const int grid = tabled ? ceil_div(sa.n_wg, 8 * n_qg) * 8 * n_qg : ceil_div(sa.n_wg, 8) * 8;
        if (tm.begin(K)) return -1;
        if (tabled) {
            WorkTableArgs wa{};
            wa.n_cmp = n_cmp; wa.n_query = n_query; wa.B = p->B; wa.T = p->T; wa.max_n_cmp = p->max_n_cmp;
            wa.scan_table = reinterpret_cast<int32_t*>(ws + lo.off_cmp_table);
            wa.scan_items_max = lo.cmp_items_max; wa.scan_slices_cap = pl.n_cmp_chunks;
            wa.imp_table = lo.imp_items_max ? reinterpret_cast<int32_t*>(ws + lo.off_imp_table) : nullptr;
            wa.imp_items_max = lo.imp_items_max;
            hipLaunchKernelGGL(k_work_table, dim3(1), dim3(kThreads), 0, stream, wa);
        }
        for (int r = 0; r < reps; ++r) {
#define SSV_LAUNCH_STREAM(NRT_, ROLES_) SSV_LAUNCH(K, (k_stream<BF16, DK, DV, NRT_, ROLES_>), grid, lds_stream, sa)
            if (C * lo.H_g > 64) {
                if (roles == kRolesAll) SSV_LAUNCH_STREAM(2, kRolesAll);
                else if (roles == kRolesSlc) SSV_LAUNCH_STREAM(2, kRolesSlc);
                else if (roles == kRolesWinSlc) SSV_LAUNCH_STREAM(2, kRolesWinSlc);
                else SSV_LAUNCH_STREAM(2, kRolesCmpWin);
            } else {
                if (roles == kRolesAll) SSV_LAUNCH_STREAM(1, kRolesAll);
                else if (roles == kRolesSlc) SSV_LAUNCH_STREAM(1, kRolesSlc);
                else if (roles == kRolesWinSlc) SSV_LAUNCH_STREAM(1, kRolesWinSlc);
                else if (roles == kRolesCmp) SSV_LAUNCH_STREAM(1, kRolesCmp);
                else if (roles == kRolesWin) SSV_LAUNCH_STREAM(1, kRolesWin);
                else SSV_LAUNCH_STREAM(1, kRolesCmpWin);
            }
#undef SSV_LAUNCH_STREAM
        }
        return (hipGetLastError() == hipSuccess && !tm.end(K)) ? 0 : -1;
    };

    // the compressed scan in the matrix-core kernel: partial-state slots [0, n_cmp_chunks), groups of C_scan queries
    auto launch_scan32 = [&]() -> int {
        if constexpr (BF16) {
            Scan32Args ca{};
            ca.q = sa.q; ca.kc = sa.kc; ca.vc = sa.vc; ca.seq_lens = seq_lens; ca.n_cmp = n_cmp; ca.n_query = n_query; ca.parents = parents;
            ca.part_stats = part_stats; ca.part_acc = part_acc;
            ca.B = p->B; ca.T = p->T; ca.H = p->H; ca.H_kv = p->H_kv; ca.H_g = lo.H_g; ca.C = pl.C_scan; ca.n_qg = pl.n_qg_scan;
            ca.l = p->l; ca.d = p->d; ca.max_seq_len = p->max_seq_len; ca.max_n_cmp = p->max_n_cmp; ca.scale_log2 = scale_log2;
            ca.n_chunks = pl.n_cmp_chunks;
            ca.n_ranges = lo.scan_ranges;
            ca.range_min = lo.scan_range_min;
            ca.pair_cost = kScan32PairCost;
            ca.imp_items_max = lo.imp_items_max;
            ca.imp_table = lo.imp_items_max ? reinterpret_cast<int32_t*>(ws + lo.off_imp_table) : nullptr;
            ca.n_wg = lo.scan_balanced ? lo.scan_ranges * pl.n_qg_scan : p->B * p->H_kv * pl.n_qg_scan * pl.n_cmp_chunks;
            ca.min_tiles = ca.n_wg > kScan32Wgs ? kScan32MinTilesMultiRound : 1;
            ca.rows_total = lo.rows_total;
            for (int j = 0; j < 3; ++j) { ca.kc_s[j] = sa.kc_s[j]; ca.vc_s[j] = sa.vc_s[j]; ca.q_s[j] = lo.q_s[j]; }
            if (pl.C_scan * lo.H_g > Scan32Cfg<DK, DV>::ROWS) return -1;      // (cannot happen: make_layout bounds C_scan)
            const int grid = ceil_div(ca.n_wg, 8) * 8;
            if (tm.begin(SSV_K_STREAM_A)) return -1;
            for (int r = 0; r < reps; ++r) {
                if (lo.scan_balanced) SSV_LAUNCH_T(SSV_K_STREAM_A, (k_scan32<DK, DV, true>), grid, kScan32Threads, (Scan32Cfg<DK, DV>::LDS), ca);
                else SSV_LAUNCH_T(SSV_K_STREAM_A, (k_scan32<DK, DV, false>), grid, kScan32Threads, (Scan32Cfg<DK, DV>::LDS), ca);
            }
            return (hipGetLastError() == hipSuccess && !tm.end(SSV_K_STREAM_A)) ? 0 : -1;
        } else {
            return -1;
        }
    };

    // routing of a refresh call: normalised head-summed probabilities, then (unless the selected-branch launch does
    // it) block importance + top-n
    auto launch_routing = [&]() -> int {
        ImportanceArgs ia{};
        ia.q = sa.q; ia.kc = sa.kc; ia.seq_lens = seq_lens; ia.n_cmp = n_cmp; ia.n_query = n_query; ia.parents = parents;
        ia.part_stats = part_stats; ia.colsum = colsum;
        ia.B = p->B; ia.T = p->T; ia.H = p->H; ia.H_kv = p->H_kv; ia.H_g = lo.H_g; ia.C = lo.imp_C; ia.n_qg = lo.imp_n_qg;
        ia.share = pl.share_group;
        ia.l = p->l; ia.d = p->d; ia.max_seq_len = p->max_seq_len; ia.max_n_cmp = p->max_n_cmp; ia.scale_log2 = scale_log2;
        ia.n_cmp_chunks = pl.n_cmp_chunks; ia.n_imp_chunks = lo.n_imp_chunks;
        ia.n_wg = p->B * p->H_kv * lo.imp_n_qg * lo.n_imp_chunks; ia.nc_pitch = lo.nc_pitch; ia.rows_total = lo.rows_total;
        if (lo.imp_items_max) {
            ia.work_table = reinterpret_cast<const int32_t*>(ws + lo.off_imp_table);
            ia.n_wg = lo.imp_items_max * p->H_kv * lo.imp_n_qg;
        }
        for (int j = 0; j < 3; ++j) { ia.kc_s[j] = sa.kc_s[j]; ia.q_s[j] = lo.q_s[j]; }
        const int grid_i = ceil_div(ia.n_wg, 8) * 8;
        if (tm.begin(SSV_K_IMPORTANCE)) return -1;
        using IK = ImportanceKernels<BF16, DK>;
        const auto imp_kernel = reinterpret_cast<void (*)(ImportanceArgs)>(const_cast<void*>(IK::fn(lo.H_g == 16 ? 16 : (lo.H_g >= 4 ? 4 : 1), lo.imp_rw)));
        for (int r = 0; r < reps; ++r) SSV_LAUNCH_T(SSV_K_IMPORTANCE, imp_kernel, grid_i, 64 * IK::waves(lo.H_g == 16 ? 16 : (lo.H_g >= 4 ? 4 : 1), lo.imp_rw), IK::LDS, ia);
        if (hipGetLastError() != hipSuccess || tm.end(SSV_K_IMPORTANCE)) return -1;

        sa.colsum = colsum; sa.sel_out = sel_idx; sa.nc_pitch = lo.nc_pitch; sa.l_sel = p->l_sel; sa.n_init = p->n_init;
        sa.n_local = p->n_local; sa.max_blocks = lo.max_blocks; sa.share = pl.share_group;
        sa.fused_topn = pl.topn_in_slc;
        if (!sa.fused_topn) {
            TopnArgs ta{};
            ta.colsum = colsum; ta.seq_lens = seq_lens; ta.n_cmp = n_cmp; ta.n_query = n_query; ta.parents = parents;
            ta.sel_idx = sel_idx; ta.B = p->B; ta.T = p->T; ta.H_kv = p->H_kv;
            ta.max_seq_len = p->max_seq_len; ta.max_n_cmp = p->max_n_cmp;
            ta.l = p->l; ta.d = p->d; ta.l_sel = p->l_sel; ta.n_sel = p->n_sel; ta.n_init = p->n_init; ta.n_local = p->n_local;
            ta.nc_pitch = lo.nc_pitch; ta.max_blocks = lo.max_blocks; ta.share = ia.share;
            const size_t lds_topn = topn_lds_bytes(lo.max_blocks);
            if (lds_topn > 64 * 1024 &&
                hipFuncSetAttribute((const void*)k_topn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_topn) != hipSuccess)
                return -1;
            if (tm.begin(SSV_K_TOPN)) return -1;
            for (int r = 0; r < reps; ++r)
                SSV_LAUNCH(SSV_K_TOPN, k_topn, p->B * p->T * p->H_kv, lds_topn, ta);
            if (hipGetLastError() != hipSuccess || tm.end(SSV_K_TOPN)) return -1;
        }
        return 0;
    };

    CombineArgs ca{};
    ca.part_stats = part_stats; ca.part_acc = part_acc; ca.gates = gates; ca.n_query = n_query; ca.out = out;
    ca.T = p->T; ca.H = p->H; ca.n_cmp_chunks = pl.n_cmp_chunks; ca.n_win_splits = pl.n_win_splits;
    ca.n_slc_splits = pl.n_slc_splits; ca.rows_total = lo.rows_total;
    ca.br_lo = 0; ca.br_hi = 3; ca.use_gates = 1;
    for (int j = 0; j < 3; ++j) ca.out_s[j] = lo.out_s[j];
    const int rows_per_wg = kThreads / (DV / 4);
    const int grid_rows = (int)((lo.rows_total + rows_per_wg - 1) / rows_per_wg);
    const int n_scan_slots = pl.n_cmp_chunks + pl.n_win_splits;
    if (tm.begin(SSV_T_EVENT_PAIR, true) || tm.end(SSV_T_EVENT_PAIR, true)) return SSV_ELAUNCH;   // empty pair: the overhead itself

    if (lo.unfused) {
        // The execution the fused path replaces: every query on its own (C = 1), one launch per branch; each branch's
        // partial states are merged, normalised and written to scratch in the storage type; a gate kernel reads the
        // three branch outputs back.  In a refresh call the indices go through sel_idx in HBM (separate top-n launch).
        char* branch = ws + lo.off_branch;
        auto branch_out = [&](int K, int br) -> int {
            CombineArgs ba = ca;
            ba.out = branch + (size_t)br * lo.branch_bytes;
            ba.out_s[0] = (int64_t)p->T * p->H * DV * es; ba.out_s[1] = (int64_t)p->H * DV * es; ba.out_s[2] = (int64_t)DV * es;
            ba.br_lo = br; ba.br_hi = br + 1; ba.use_gates = 0;
            if (tm.begin(K)) return -1;
            for (int r = 0; r < reps; ++r) SSV_LAUNCH(K, (k_combine_rows<BF16, DV>), grid_rows, 0, ba);
            return (hipGetLastError() == hipSuccess && !tm.end(K)) ? 0 : -1;
        };
        if (launch_stream(SSV_K_STREAM_A, kRolesCmp, 0, pl.n_cmp_chunks, 1, p->T) || branch_out(SSV_K_OUT_CMP, 0)) return SSV_ELAUNCH;
        if (p->mode != SSV_REUSE && launch_routing()) return SSV_ELAUNCH;
        sa.fused_topn = 0;
        if (launch_stream(SSV_K_STREAM_B, kRolesSlc, n_scan_slots, pl.n_slc_splits, 1, p->T) || branch_out(SSV_K_OUT_SLC, 1)) return SSV_ELAUNCH;
        if (launch_stream(SSV_K_STREAM_W, kRolesWin, pl.n_cmp_chunks, pl.n_win_splits, 1, p->T) || branch_out(SSV_K_OUT_WIN, 2)) return SSV_ELAUNCH;
        GateArgs ga{};
        ga.o_cmp = branch; ga.o_slc = branch + lo.branch_bytes; ga.o_win = branch + 2 * lo.branch_bytes;
        ga.gates = gates; ga.n_query = n_query; ga.out = out; ga.T = p->T; ga.H = p->H; ga.rows_total = lo.rows_total;
        for (int j = 0; j < 3; ++j) ga.out_s[j] = lo.out_s[j];
        if (tm.begin(SSV_K_COMBINE)) return SSV_ELAUNCH;
        for (int r = 0; r < reps; ++r) SSV_LAUNCH(SSV_K_COMBINE, (k_gate<BF16, DV>), grid_rows, 0, ga);
        if (hipGetLastError() != hipSuccess || tm.end(SSV_K_COMBINE)) return SSV_ELAUNCH;
        return SSV_OK;
    }

    if (lo.scan32) {
        if (launch_scan32()) return SSV_ELAUNCH;
        if (p->mode != SSV_REUSE && launch_routing()) return SSV_ELAUNCH;
        sa.joint = lo.joint_parts;
        if (launch_stream(SSV_K_STREAM_B, kRolesWinSlc, pl.n_cmp_chunks, lo.joint_parts ? lo.joint_parts : pl.n_win_splits + pl.n_slc_splits, pl.C,
                          pl.n_qg))
            return SSV_ELAUNCH;
    } else if (lo.one_launch) {
        if (launch_stream(SSV_K_STREAM_A, kRolesAll, 0, pl.n_slots, pl.C, pl.n_qg)) return SSV_ELAUNCH;
    } else {
        if (launch_stream(SSV_K_STREAM_A, kRolesCmpWin, 0, n_scan_slots, pl.C_scan, pl.n_qg_scan)) return SSV_ELAUNCH;
        if (p->mode != SSV_REUSE && launch_routing()) return SSV_ELAUNCH;
        if (launch_stream(SSV_K_STREAM_B, kRolesSlc, n_scan_slots, pl.n_slc_splits, pl.C, pl.n_qg)) return SSV_ELAUNCH;
    }
    // few slices per row: thread groups own rows; many slices: one workgroup per row, slices in parallel
    // (13..16 slices: thread groups only where there are rows enough to fill the chip with them)
    const bool by_rows = pl.n_slots <= 12 || (pl.n_slots <= kCombineRowsMaxSlots && lo.rows_total >= 4096);
    // partial states of tens of megabytes: the streaming form (statistics first, then only the accumulators that count)
    const bool eager = (int64_t)pl.n_slots * lo.rows_total * (DV + 2) * 4 <= (int64_t)40 << 20;
    // the streaming combine: persistent workgroups, every one the same number of batches of rows
    const int n_batches = grid_rows, rounds = ceil_div(n_batches, kCombineStreamWgs);
    const int grid_stream = ceil_div(n_batches, rounds);
    if (tm.begin(SSV_K_COMBINE)) return SSV_ELAUNCH;
    for (int r = 0; r < reps; ++r) {
        if (by_rows && eager) SSV_LAUNCH(SSV_K_COMBINE, (k_combine_rows<BF16, DV>), grid_rows, 0, ca);
        else if (by_rows) SSV_LAUNCH(SSV_K_COMBINE, (k_combine_stream<BF16, DV>), grid_stream, 0, ca);
        else SSV_LAUNCH(SSV_K_COMBINE, (k_combine_slices<BF16, DV>), (int)lo.rows_total, 0, ca);
    }
    if (hipGetLastError() != hipSuccess || tm.end(SSV_K_COMBINE)) return SSV_ELAUNCH;
    return SSV_OK;
}

int verify_impl(const void* q, const void* k, const void* v, const void* kc, const void* vc, const float* gates,
                const int32_t* seq_lens, const int32_t* n_cmp, const int32_t* n_query, const int32_t* parents,
                const ssv_nsa_params* p, void* out, int32_t* sel_idx, void* workspace, size_t workspace_bytes,
                void* stream, float* kernel_ms, int repeats, bool timed) {
    // the parameter checks come first and are the ones ssv_nsa_plan_query and ssv_nsa_workspace_bytes run
    Layout lo;
    const int rc = make_layout(p, &lo);
    if (rc != SSV_OK) return rc;
    if (!q || !k || !v || !kc || !vc || !gates || !seq_lens || !n_cmp || !out || !sel_idx) return SSV_EINVAL;
    if (timed && (!kernel_ms || repeats < 1 || repeats > 1000)) return SSV_EINVAL;
    const void* aligned16[] = {q, k, v, kc, vc, out};
    for (const void* ptr : aligned16)
        if (reinterpret_cast<uintptr_t>(ptr) % 16) return SSV_EINVAL;
    if (!workspace || reinterpret_cast<uintptr_t>(workspace) % 256 || workspace_bytes < lo.total) return SSV_EWORKSPACE;

    Timer tm;
    tm.on = timed;
    tm.repeats = timed ? repeats : 1;
    tm.stream = (hipStream_t)stream;
    int res = SSV_EUNSUPPORTED;
#define SSV_DISPATCH(BF, DK, DV)                                                                                     \
    if (p->dtype == ((BF) ? SSV_BF16 : SSV_F32) && p->d_k == (DK) && p->d_v == (DV))                                 \
        res = launch_all<BF, DK, DV>(q, k, v, kc, vc, gates, seq_lens, n_cmp, n_query, parents, p, out, sel_idx,      \
                                     (char*)workspace, lo, (hipStream_t)stream, tm);
    SSV_DISPATCH(true, 192, 128)
    SSV_DISPATCH(true, 128, 128)
    SSV_DISPATCH(true, 64, 64)
    SSV_DISPATCH(false, 64, 64)
#undef SSV_DISPATCH
    if (timed) {
        const int frc = tm.finish(kernel_ms);
        if (res == SSV_OK && frc) res = SSV_ELAUNCH;
    }
    return res;
}

}  // namespace

extern "C" {

int ssv_nsa_supported(int32_t dtype, int32_t d_k, int32_t d_v) {
    for (const Shape& s : kShapes)
        if (s.dtype == dtype && s.d_k == d_k && s.d_v == d_v) return 1;
    return 0;
}

int ssv_nsa_plan_query(const ssv_nsa_params* p, ssv_nsa_plan* plan) {
    if (!plan) return SSV_EINVAL;
    Layout lo;
    const int rc = make_layout(p, &lo);
    if (rc == SSV_OK) *plan = lo.plan;
    return rc;
}

size_t ssv_nsa_workspace_bytes(const ssv_nsa_params* p) {
    Layout lo;
    return make_layout(p, &lo) == SSV_OK ? lo.total : 0;
}

int ssv_nsa_verify(const void* q, const void* k, const void* v, const void* k_cmp, const void* v_cmp,
                   const float* gates, const int32_t* seq_lens, const int32_t* n_cmp, const int32_t* n_query,
                   const int32_t* tree_parents, const ssv_nsa_params* p, void* out, int32_t* sel_idx, void* workspace,
                   size_t workspace_bytes, void* stream) {
    return verify_impl(q, k, v, k_cmp, v_cmp, gates, seq_lens, n_cmp, n_query, tree_parents, p, out, sel_idx, workspace,
                       workspace_bytes, stream, nullptr, 1, false);
}

int ssv_nsa_verify_static(const void* q, const void* k, const void* v, const void* k_cmp, const void* v_cmp,
                          const float* gates, const int32_t* seq_lens, const int32_t* n_cmp, const int32_t* n_query,
                          const int32_t* tree_parents, const ssv_nsa_params* p, void* out, int32_t* sel_idx, void* stream) {
    Layout lo;
    const int rc = make_layout(p, &lo);
    if (rc != SSV_OK) return rc;
    if (lo.total > (size_t)SSV_STATIC_SCRATCH_BYTES) return SSV_ESTATIC;
    // address of the current device's copy of the array, looked up once per device
    static std::atomic<void*> scratch_ptr[kMaxDevices];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return SSV_ELAUNCH;
    void* ptr = scratch_ptr[dev].load(std::memory_order_acquire);
    if (!ptr) {
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return SSV_ELAUNCH;
        scratch_ptr[dev].store(ptr, std::memory_order_release);     // (two host threads racing here store the same address)
    }
    return verify_impl(q, k, v, k_cmp, v_cmp, gates, seq_lens, n_cmp, n_query, tree_parents, p, out, sel_idx, ptr,
                       (size_t)SSV_STATIC_SCRATCH_BYTES, stream, nullptr, 1, false);
}

int ssv_nsa_verify_timed(const void* q, const void* k, const void* v, const void* k_cmp, const void* v_cmp,
                         const float* gates, const int32_t* seq_lens, const int32_t* n_cmp, const int32_t* n_query,
                         const int32_t* tree_parents, const ssv_nsa_params* p, void* out, int32_t* sel_idx,
                         void* workspace, size_t workspace_bytes, void* stream, int repeats, float* kernel_ms) {
    return verify_impl(q, k, v, k_cmp, v_cmp, gates, seq_lens, n_cmp, n_query, tree_parents, p, out, sel_idx, workspace,
                       workspace_bytes, stream, kernel_ms, repeats, true);
}

int ssv_nsa_compress(const void* k, const void* v, void* k_cmp, void* v_cmp, const int32_t* committed_before,
                     const int32_t* committed_after, int32_t* n_cmp, const ssv_cmp_params* p, void* stream) {
    if (!k || !v || !k_cmp || !v_cmp || !committed_after || !n_cmp || !p) return SSV_EINVAL;
    if (p->B < 1 || p->H_kv < 1 || p->d_k < 1 || p->d_v < 1 || p->l < 1 || p->d < 1 || p->l % p->d) return SSV_EINVAL;
    if (p->dtype != SSV_F32 && p->dtype != SSV_BF16) return SSV_EINVAL;
    if (p->max_new_rows < 1 || p->kv_capacity < 0 || p->cmp_capacity < 1) return SSV_EINVAL;
    const int es = p->dtype == SSV_BF16 ? 2 : 4;
    if ((p->d_k * es) % 16 || (p->d_v * es) % 16) return SSV_EINVAL;
    const int64_t* strides[4] = {p->k_stride, p->v_stride, p->kc_stride, p->vc_stride};
    const int dims[4] = {p->d_k, p->d_v, p->d_k, p->d_v};
    for (int a = 0; a < 4; ++a)
        for (int j = 0; j < 3; ++j) {
            if (strides[a][j] < 0 || (strides[a][j] * es) % 16) return SSV_EINVAL;
            if (j == 2 && strides[a][j] < dims[a]) return SSV_EINVAL;
        }
    const void* aligned16[] = {k, v, k_cmp, v_cmp};
    for (const void* ptr : aligned16)
        if (reinterpret_cast<uintptr_t>(ptr) % 16) return SSV_EINVAL;
    const int ratio = p->l / p->d;
    if (ratio > 64 || p->d_k > 1024 || p->d_v > 1024) return SSV_EUNSUPPORTED;

    CompressArgs ca{};
    ca.k = (const char*)k; ca.v = (const char*)v; ca.kc = (char*)k_cmp; ca.vc = (char*)v_cmp;
    ca.before = committed_before; ca.after = committed_after; ca.n_cmp = n_cmp;
    ca.B = p->B; ca.H_kv = p->H_kv; ca.l = p->l; ca.d = p->d; ca.ratio = ratio;
    // 32 chunks per workgroup: with 16 or 24 column groups per row the chunk tasks fill whole passes of 256 threads
    ca.rows_per_wg = std::min(std::max(1, 33 - ratio), p->max_new_rows); ca.cap = p->cmp_capacity; ca.kv_cap = p->kv_capacity;
    ca.max_new = p->max_new_rows;
    ca.k_groups = p->d_k * es / 16; ca.v_groups = p->d_v * es / 16;
    ca.inv_l = 1.0f / (float)p->l;
    for (int j = 0; j < 3; ++j) {
        ca.k_s[j] = p->k_stride[j] * es; ca.v_s[j] = p->v_stride[j] * es;
        ca.kc_s[j] = p->kc_stride[j] * es; ca.vc_s[j] = p->vc_stride[j] * es;
    }
    const size_t lds = (size_t)(ca.rows_per_wg + ratio - 1) * std::max(p->d_k, p->d_v) * sizeof(float);
    if (lds > 64 * 1024) return SSV_EUNSUPPORTED;
    const dim3 grid(ceil_div(p->max_new_rows, ca.rows_per_wg), p->B * p->H_kv, 2);
    if (grid.y > 65535) return SSV_EUNSUPPORTED;
    if (p->dtype == SSV_BF16) hipLaunchKernelGGL((k_compress<true>), grid, dim3(kThreads), lds, (hipStream_t)stream, ca);
    else hipLaunchKernelGGL((k_compress<false>), grid, dim3(kThreads), lds, (hipStream_t)stream, ca);
    return hipGetLastError() == hipSuccess ? SSV_OK : SSV_ELAUNCH;
}

void ssv_guard_default_config(ssv_guard_config* cfg) {
    if (!cfg) return;
    cfg->alpha = 0.40; cfg->ratio = 0.85; cfg->warmup_steps = 8; cfg->patience = 5; cfg->max_transitions = 2;
    cfg->early_steps = 0;
}

int ssv_guard_init(ssv_guard_state* state, const ssv_guard_config* cfg, const double* expected, const uint8_t* valid,
                   int32_t n) {
    return ssv::guard_init(state, cfg, expected, valid, n);
}

int ssv_guard_observe(ssv_guard_state* state, double accepted_tokens, double step_latency) {
    return ssv::guard_observe(state, accepted_tokens, step_latency);
}

int ssv_tree_flatten(const int32_t* parents, int32_t n, int32_t order, int32_t* perm, int32_t* new_parents) {
    return ssv::tree_flatten(parents, n, order, perm, new_parents);
}

const char* ssv_nsa_strerror(int code) {
    switch (code) {
        case SSV_OK: return "ok";
        case SSV_EINVAL: return "invalid argument";
        case SSV_EUNSUPPORTED: return "shape not supported by this build";
        case SSV_EWORKSPACE: return "workspace missing, misaligned or too small";
        case SSV_ELAUNCH: return "HIP launch failed";
        case SSV_ESTATIC: return "problem needs more scratch than the static array of ssv_nsa_verify_static holds";
        default: return "unknown error";
    }
}

const char* ssv_nsa_kernel_name(int idx) {
    switch (idx) {
        case SSV_K_STREAM_A: return "k_stream (compressed scan + window; all branches in reuse mode)";
        case SSV_K_IMPORTANCE: return "k_importance";
        case SSV_K_TOPN: return "k_topn";
        case SSV_K_STREAM_B: return "k_stream (selected blocks, merged schedule)";
        case SSV_K_COMBINE: return "k_combine";
        case SSV_K_STREAM_W: return "k_stream (window branch alone; unfused execution)";
        case SSV_K_OUT_CMP: return "k_combine_rows (compressed branch output to scratch; unfused execution)";
        case SSV_K_OUT_SLC: return "k_combine_rows (selected branch output to scratch; unfused execution)";
        case SSV_K_OUT_WIN: return "k_combine_rows (window branch output to scratch; unfused execution)";
        default: return "";
    }
}

int ssv_nsa_version(void) { return 2; }

}  // extern "C"

