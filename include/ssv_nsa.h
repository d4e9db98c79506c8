/*
 * ssv_nsa.h -- C ABI of the MI355X (gfx950) NSA speculative-verification attention library.
 *
 * One call scores a batch of speculative verifier queries (linear draft chains or draft
 * trees) against a long KV cache with Native Sparse Attention: compressed attention over
 * pooled KV blocks, per-GQA-group top-n block selection routed by the compressed
 * probabilities, selected-block attention and sliding-window attention, combined by
 * per-branch gates (paper Section 2.2).  Selected blocks are loaded once per group of
 * verifier queries as the sorted, de-duplicated union of their index sets and masked per
 * query (exact merged schedule, Section 4.2); queries are grouped C at a time so that the
 * heads of a GQA group times C queries form the rows of the matrix tiles (Section 4.1).
 * SSV_REFRESH computes and writes the selected indices (routing launch followed by the
 * downstream launch, Section 5.1); SSV_REUSE reads them and skips index construction
 * (Section 5.2).  SSV_REFRESH_SHARED is the approximate shared-index variant (Section 4.3):
 * one representative query per group of C routes for the whole group.
 *
 * Conventions
 *  - Every data pointer is DEVICE memory owned by the caller; `p`, return codes and
 *    `kernel_ms` are HOST.  The library allocates nothing; scratch comes from `workspace`.  Nothing in the call path reads
 *    the process environment: every choice is a field of the parameter struct, 0 meaning automatic.
 *  - All work is enqueued on `stream` (a hipStream_t passed as void*); ssv_nsa_verify never
 *    synchronises.  Nothing is launched when an error code is returned.
 *  - Per sequence b: L = seq_lens[b] committed tokens occupy KV slots 0..L-1 (slot =
 *    position); draft token i (flattened order) occupies slot L+i.  parents[b*T+i] is -1
 *    (child of the last committed token) or the index (< i) of the parent draft token.
 *    Draft token i sees the L committed tokens, itself and its ancestors.
 *  - Layout: q [B,T,H,d_k] and out [B,T,H,d_v], contiguous unless q_stride / out_stride say
 *    otherwise (elements: batch, query, head; the feature dimension is contiguous); k, v, k_cmp,
 *    v_cmp addressed as base + b*stride[0] + kv_head*stride[1] + row*stride[2] (+ contiguous
 *    feature), strides in elements; gates [B,T,H,3] float32 in the order (compressed, selected, window);
 *    sel_idx [B,T,H_kv,n_sel] int32, ascending, padded with -1.
 */
#ifndef SSV_NSA_H
#define SSV_NSA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SSV_OK            0
#define SSV_EINVAL       -1   /* null pointer, inconsistent or out-of-range parameter */
#define SSV_EUNSUPPORTED -2   /* valid NSA problem, but a shape this build has no kernel for */
#define SSV_EWORKSPACE   -3   /* workspace missing, misaligned or smaller than ssv_nsa_workspace_bytes */
#define SSV_ELAUNCH      -4   /* the HIP runtime reported an error when enqueueing */
#define SSV_ESTATIC      -5   /* ssv_nsa_verify_static: the problem needs more scratch than SSV_STATIC_SCRATCH_BYTES */

#define SSV_F32  0
#define SSV_BF16 1

#define SSV_REFRESH 0
#define SSV_REUSE   1
#define SSV_REFRESH_SHARED 2  /* approximate: every group of C queries uses its representative's indices */

#define SSV_MAX_T 128         /* verifier queries per sequence */

/* ssv_nsa_params.exec: how the call is executed (never changes what is computed beyond rounding) */
#define SSV_EXEC_FUSED   0    /* grouped queries, merged schedule, branches fused: the path this library is built for */
#define SSV_EXEC_UNFUSED 1    /* the execution the fused path replaces (Section 5, the original NSA kernel structure; the
                                 baseline side of the ratios of Section 7.3): every verifier query on its own (no
                                 grouping, no merged schedule), one launch per branch, each branch output normalised and
                                 written to scratch in the storage type, then read back by a separate gate kernel */

/* ssv_nsa_params.topn_home: where the top-n selection of a refresh call runs */
#define SSV_TOPN_AUTO     0   /* inside the selected-branch launch when that launch has at most one workgroup per CU */
#define SSV_TOPN_SEPARATE 1   /* always a launch of its own */
#define SSV_TOPN_IN_SLC   2   /* inside the selected-branch launch whenever its scratch fits the tile buffers */

/* ssv_nsa_params.scan_kernel: which kernel scans the compressed cache */
#define SSV_SCAN_AUTO   0     /* the matrix-core scan where a KV head has 192 rows or more and the scan runs for several
                                 tiles per workgroup, else the streaming kernel */
#define SSV_SCAN_STREAM 1     /* the streaming kernel (64 or 128 rows per workgroup, two workgroups per CU) */
#define SSV_SCAN_MATRIX 2     /* the matrix-core scan (bf16 only: 256 rows per workgroup, one workgroup per CU; the window
                                 branch then runs in the selected-branch launch) */
#define SSV_SCAN_STREAM_TABLE 3 /* the streaming kernel with its slices taken from a work table built on the device from
                                 the lengths (what SSV_SCAN_AUTO and SSV_SCAN_STREAM do for long scans of mixed-length
                                 batches), whenever the batch and the launch allow it (SSV_EXEC_FUSED only) */

/* kernels of one call, in launch order (indices into kernel_ms of ssv_nsa_verify_timed) */
#define SSV_K_STREAM_A  0     /* refresh: compressed scan + window;  reuse: compressed + window (+ selected, unless
                                 SSV_K_STREAM_B is launched); with plan.scan_matrix: the compressed scan alone */
#define SSV_K_IMPORTANCE 1    /* refresh only: normalised compressed probabilities summed over the group's heads */
#define SSV_K_TOPN      2     /* refresh only: block importance + top-n selection; not launched (time 0) when the
                                 selection runs inside SSV_K_STREAM_B, which it does when that launch has at most
                                 one workgroup per CU */
#define SSV_K_STREAM_B  3     /* selected-block attention over the merged schedule: refresh, and reuse when the scans
                                 of SSV_K_STREAM_A use larger query groups than the selected branch (plan.C_scan > C);
                                 with plan.scan_matrix: selected blocks + window */
#define SSV_K_COMBINE   4     /* merge of split partial states + gated combination */
#define SSV_K_STREAM_W  5     /* SSV_EXEC_UNFUSED only: the window branch as a launch of its own (SSV_K_STREAM_A then is
                                 the compressed branch alone) */
#define SSV_K_OUT_CMP   6     /* SSV_EXEC_UNFUSED only: merge of the compressed branch's partial states, branch output
                                 written to scratch; SSV_K_OUT_SLC, SSV_K_OUT_WIN: the same for the other two
                                 branches; SSV_K_COMBINE then is the gate kernel that reads the three back */
#define SSV_K_OUT_SLC   7
#define SSV_K_OUT_WIN   8
#define SSV_NUM_KERNELS 9
#define SSV_T_EVENT_PAIR 9    /* ssv_nsa_verify_timed only: duration of an empty event pair (measurement overhead) */
#define SSV_NUM_TIMINGS 10

typedef struct ssv_nsa_params {
    int32_t B;            /* sequences in the batch */
    int32_t T;            /* verifier queries per sequence (row capacity), 1..SSV_MAX_T */
    int32_t H, H_kv;      /* query heads, KV heads; H_g = H / H_kv in {1,2,4,8,16} */
    int32_t d_k, d_v;     /* head dims of K and V; supported (dtype,d_k,d_v): see ssv_nsa_supported */
    int32_t l, d;         /* compression block length and stride (l % d == 0) */
    int32_t l_sel;        /* selection block size l' (this build: 64) */
    int32_t n_sel;        /* selected blocks per query, forced ones included (<= 32) */
    int32_t w;            /* sliding window, in positions, ending at and including the query */
    int32_t n_init;       /* forced leading blocks */
    int32_t n_local;      /* forced blocks ending at the block of the query's own slot */
    int32_t dtype;        /* SSV_F32 or SSV_BF16: type of q, k, v, k_cmp, v_cmp, out */
    int32_t mode;         /* SSV_REFRESH, SSV_REFRESH_SHARED: sel_idx is written; SSV_REUSE: sel_idx is read */
    int32_t group_size;   /* SSV_REFRESH, SSV_REUSE: C, verifier queries per workgroup (C <= 64, C * H_g <= 128); 0 = auto
                             (C * H_g <= 64); never changes the result.  SSV_REFRESH_SHARED: queries per index-sharing
                             group (1..T; 0 = the automatic C); the workgroup grouping is then the automatic one */
    float   scale;        /* softmax scale; 0 => 1/sqrt(d_k) */
    int32_t max_seq_len;  /* host-side upper bound on seq_lens[b] (sizes grids and scratch); k and v hold at least
                             max_seq_len + T rows per (sequence, KV head); larger seq_lens[b] are clamped to it */
    int32_t max_n_cmp;    /* host-side upper bound on n_cmp[b] = rows of k_cmp / v_cmp per (sequence, KV head); larger
                             n_cmp[b] are clamped to it */
    int32_t avg_seq_len;  /* host-side hint: mean of seq_lens[b] (balances splits of mixed-length batches); 0 = max_seq_len */
    int32_t scan_group_size; /* queries per workgroup in the launch of the compressed and window scans (<= 64,
                             times H_g <= 128); 0 = automatic: group_size if that is given, else up to 128 rows where
                             the scans keep the chip busy for several rounds; never changes the result */
    int64_t k_stride[3], v_stride[3], kc_stride[3], vc_stride[3];  /* elements: batch, KV head, row */
    int64_t q_stride[3], out_stride[3];  /* elements: batch, query, head; all zero = contiguous [B,T,H,d] */
    int32_t exec;         /* SSV_EXEC_FUSED or SSV_EXEC_UNFUSED (SSV_REFRESH and SSV_REUSE only; group_size and
                             scan_group_size must be 0 or 1 there) */
    int32_t topn_home;    /* SSV_TOPN_AUTO, SSV_TOPN_SEPARATE or SSV_TOPN_IN_SLC; never changes the result */
    int32_t max_slice_tiles; /* upper bound on the 64-row tiles one workgroup streams when a launch needs several
                             rounds of workgroups (2..64; 0 = automatic: 32); never changes the result */
    int32_t imp_rows;     /* rows (routed queries x heads of a group) per workgroup in the importance pass of a refresh
                             call: 64, 128 or 256; 0 = automatic (more than 64 where a KV head has that many rows and
                             the pass runs for several tiles per workgroup); never changes the result */
    int32_t scan_kernel;  /* SSV_SCAN_AUTO, SSV_SCAN_STREAM, SSV_SCAN_STREAM_TABLE or SSV_SCAN_MATRIX (SSV_EXEC_FUSED,
                             SSV_BF16 only; with it scan_group_size may reach 256 / H_g); never changes the result
                             beyond rounding */
} ssv_nsa_params;

/* How one call is cut into workgroups (host-side planning; filled by ssv_nsa_plan). */
typedef struct ssv_nsa_plan {
    int32_t C;                /* verifier queries per group */
    int32_t n_qg;             /* query groups per (sequence, KV head) */
    int32_t rows_per_wg;      /* C * H_g */
    int32_t n_cmp_chunks;     /* workgroups splitting the compressed scan of one group */
    int32_t tiles_per_chunk;  /* 64-row tiles of k_cmp/v_cmp per such workgroup */
    int32_t n_win_splits;     /* workgroups splitting the window tiles of one group */
    int32_t n_slc_splits;     /* workgroups splitting the merged selected-block schedule of one group */
    int32_t min_tiles_per_split;
    int32_t n_slots;          /* partial softmax states per output row = sum of the three above */
    int32_t max_sched_entries;/* capacity of the merged schedule of one group */
    int32_t share_group;      /* SSV_REFRESH_SHARED: queries per index-sharing group; 0 in the other modes */
    int32_t C_scan;           /* queries per group in the launch of the compressed and window scans (>= C: every
                                 query of a sequence reads the same rows there, so larger groups only save loads;
                                 the merged schedule of the selected branch grows with its group) */
    int32_t n_qg_scan;        /* such groups per (sequence, KV head) */
    int32_t topn_in_slc;      /* refresh: 1 if the top-n selection runs inside the selected-branch launch, else 0 */
    int32_t n_imp_chunks;     /* refresh: workgroups splitting the importance pass over k_cmp of one query group */
    int32_t imp_rows;         /* refresh: rows per workgroup in the importance pass (64, 128 or 256) */
    int32_t n_launches;       /* kernel launches of one call */
    int32_t scan_matrix;      /* 1 if the compressed scan runs in the matrix-core kernel (then C_scan counts its groups of
                                 up to 256 rows and the window branch runs in the selected-branch launch), else 0 */
    int64_t workspace_bytes;
} ssv_nsa_plan;

/*
 * NSA verification attention (Section 2.2 branches; Section 4.1-4.2 grouping and merged schedule;
 * Section 5.1 refresh / Section 5.2 reuse).
 *   q, k, v, k_cmp, v_cmp, gates, out: see layout above.
 *   seq_lens [B], n_cmp [B] (compressed rows available per sequence), n_query [B] or NULL (= T each),
 *   tree_parents [B,T] or NULL (= linear chain): device int32.
 *   A compressed row c (covering slots [c*d, c*d+l)) is used by query i only if c < n_cmp[b] and all
 *   its slots are visible to i as a contiguous run from slot 0.
 *   sel_idx: written in SSV_REFRESH; read in SSV_REUSE, where negative, repeated or out-of-range
 *   entries are ignored.  Rows of queries i >= n_query[b]: out = 0, sel_idx = -1 (refresh).
 *   SSV_REFRESH_SHARED (Section 4.3): queries [m*G, (m+1)*G) of a sequence (flattened order, G = plan.share_group)
 *   form a group; its representative is the member with the largest position L + depth, the last such member if
 *   several are equally deep (the last query of the group in a chain).  Block importance and top-n run for the
 *   representative only; its index set is written to the sel_idx row of every member and every member's
 *   selected branch attends to it under the member's own visibility.  Compressed and window branches are
 *   those of SSV_REFRESH.  The result equals SSV_REUSE on the sel_idx it writes.
 *   workspace: >= ssv_nsa_workspace_bytes(p) bytes, 256-byte aligned; contents need not be preserved
 *   or initialised between calls; calls sharing a workspace must not overlap in time.
 * Returns SSV_OK or a negative SSV_E* code.
 */
int ssv_nsa_verify(const void* q, const void* k, const void* v, const void* k_cmp, const void* v_cmp,
                   const float* gates, const int32_t* seq_lens, const int32_t* n_cmp, const int32_t* n_query,
                   const int32_t* tree_parents, const ssv_nsa_params* p, void* out, int32_t* sel_idx,
                   void* workspace, size_t workspace_bytes, void* stream);

/*
 * Same computation, timed per kernel (all kernels are idempotent, so the results are those of ssv_nsa_verify); the
 * call synchronises `stream` before returning and writes the average duration of one launch of each kernel, in
 * milliseconds, to kernel_ms[SSV_NUM_TIMINGS] (host; 0 for kernels the mode does not launch).
 * repeats == 1: every kernel is launched once with start and stop events bound to the launch itself, which read
 * the dispatch's own begin and end (the duration a kernel trace shows for it).  repeats in 2..1000: every kernel
 * is launched that many times back to back between one pair of events on `stream`.
 * kernel_ms[SSV_T_EVENT_PAIR] is the duration of an event pair with nothing in between, i.e. what the event
 * mechanism adds to an interval measured the second way.
 * Measurement aid for the roofline figures (Section 7.3 reports such a per-kernel breakdown).
 */
int ssv_nsa_verify_timed(const void* q, const void* k, const void* v, const void* k_cmp, const void* v_cmp,
                         const float* gates, const int32_t* seq_lens, const int32_t* n_cmp, const int32_t* n_query,
                         const int32_t* tree_parents, const ssv_nsa_params* p, void* out, int32_t* sel_idx,
                         void* workspace, size_t workspace_bytes, void* stream, int repeats, float* kernel_ms);

/*
 * ssv_nsa_verify without a workspace argument, for callers that cannot allocate device memory (code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc): the scratch is a fixed array of
 * SSV_STATIC_SCRATCH_BYTES inside the library's device image (one copy per GPU, held until the process ends),
 * and the call allocates and frees nothing.  Same arguments, semantics and results as ssv_nsa_verify.
 * Returns SSV_ESTATIC, before anything is enqueued, when ssv_nsa_workspace_bytes(p) exceeds SSV_STATIC_SCRATCH_BYTES
 * (use ssv_nsa_verify with a workspace of the caller's for such a problem).
 * The first call on a GPU looks up that GPU's copy of the array (and, like ssv_nsa_verify, raises the kernels'
 * dynamic-LDS limit): make it outside graph capture.
 * Every call on a GPU uses that GPU's one array: calls that overlap in time on one GPU (different streams or
 * host threads) race, like calls of ssv_nsa_verify that share a workspace.  The array keeps the previous call's
 * contents; no kernel relies on them.
 */
#define SSV_STATIC_SCRATCH_BYTES (32u << 20)
int ssv_nsa_verify_static(const void* q, const void* k, const void* v, const void* k_cmp, const void* v_cmp,
                          const float* gates, const int32_t* seq_lens, const int32_t* n_cmp, const int32_t* n_query,
                          const int32_t* tree_parents, const ssv_nsa_params* p, void* out, int32_t* sel_idx,
                          void* stream);

/* Parameters of ssv_nsa_compress.  Strides in elements (sequence, KV head, row), as in ssv_nsa_params. */
typedef struct ssv_cmp_params {
    int32_t B, H_kv;
    int32_t d_k, d_v;        /* row lengths; d_k * elem and d_v * elem must be multiples of 16 bytes */
    int32_t l, d;            /* compression block length and stride (l % d == 0) */
    int32_t dtype;           /* SSV_F32 or SSV_BF16: type of k, v, k_cmp, v_cmp */
    int32_t max_new_rows;    /* host-side bound (>= 1) on the compressed rows one sequence gains in this call (sizes the grid) */
    int32_t kv_capacity;     /* rows of k / v per (sequence, KV head) */
    int32_t cmp_capacity;    /* rows (>= 1) of k_cmp / v_cmp per (sequence, KV head) */
    int64_t k_stride[3], v_stride[3], kc_stride[3], vc_stride[3];
} ssv_cmp_params;

/*
 * Compressed-cache construction, the step before ssv_nsa_verify: the compression branch aggregates committed
 * tokens into blocks of length l taken every d tokens (Section 2.2); the aggregate here is the mean of the
 * block's rows, accumulated in fp32 and rounded once to the storage type.  Compressed row c = mean of raw rows
 * [c*d, c*d + l) and exists only when all of them are committed: N(L) = 0 for L < l, else (L - l) / d + 1, so
 * draft tokens enter the compressed cache only once they are accepted (Sections 3.1 and 6 keep the raw and
 * compressed caches consistent across verification rounds).
 *   k, v (device, read), k_cmp, v_cmp (device, written): layouts of ssv_nsa_verify.
 *   committed_before [B] (device int32, or NULL = 0 everywhere: build from scratch), committed_after [B] (device
 *   int32): committed tokens per sequence before and after the update.  Rows N(before) .. N(after)-1 of every KV
 *   head are written, at most max_new_rows per sequence and never beyond cmp_capacity; committed_after is
 *   clamped to kv_capacity.  n_cmp [B] (device int32, written): rows valid after the call, min(N(after),
 *   N(before) + max_new_rows, cmp_capacity); with committed_after < committed_before (rollback) nothing is
 *   written and n_cmp shrinks to N(after).
 * All work is enqueued on `stream`; no synchronisation, no allocation.  Returns SSV_OK or a negative SSV_E* code
 * (SSV_EUNSUPPORTED: l / d > 64, or a row length above 1024 elements).
 */
int ssv_nsa_compress(const void* k, const void* v, void* k_cmp, void* v_cmp, const int32_t* committed_before,
                     const int32_t* committed_after, int32_t* n_cmp, const ssv_cmp_params* p, void* stream);

/*
 * Runtime guard of the throughput-aware planner (Section 6.3, Algorithm 1; host only, no GPU work).  A request
 * starts on the best-ranked valid strategy of its profile entry; every verification step reports its accepted-token
 * count A_t and latency T_t.  The guard smooths A_t (ema = alpha*A_t + (1-alpha)*ema, starting at the first
 * observation of a strategy); once a strategy has run warmup_steps steps, each step whose smoothed value is below
 * ratio * expected[active] counts, any other step clears the count, and patience counted steps in a row move the
 * request to the next-ranked valid strategy, restarting smoothing, warm-up and count.  After max_transitions moves
 * (or with no candidate left) a further trigger settles the request on the explored strategy with the largest
 * sum(A) / sum(T) and ends refinement; refinement also ends after early_steps steps (0 = no limit).
 * The paper's constants: alpha 0.40, warm-up 8, ratio 0.85, patience 5, two moves (ssv_guard_default_config).
 */
#define SSV_GUARD_MAX_CANDIDATES 16   /* a profile entry holds 12 ranked candidates in the paper */

typedef struct ssv_guard_config {
    double  alpha;            /* smoothing coefficient in (0, 1] */
    double  ratio;            /* fraction of the profiled expectation below which a step counts as a miss */
    int32_t warmup_steps;     /* steps of a strategy that only update the smoothed value */
    int32_t patience;         /* consecutive misses that trigger a move */
    int32_t max_transitions;  /* moves allowed per request */
    int32_t early_steps;      /* steps of the request during which refinement is active; 0 = all */
} ssv_guard_config;

/* Plain state of one request (host memory owned by the caller; no pointers inside, so it may be copied or stored). */
typedef struct ssv_guard_state {
    ssv_guard_config cfg;
    int32_t n_candidates, active, transitions, settled;
    int32_t total_steps, steps_on_active, below_streak, has_ema;
    double  ema;
    double  expected[SSV_GUARD_MAX_CANDIDATES];      /* profiled E[A] per candidate, best-ranked first */
    uint8_t valid[SSV_GUARD_MAX_CANDIDATES], explored[SSV_GUARD_MAX_CANDIDATES];
    double  sum_accepted[SSV_GUARD_MAX_CANDIDATES], sum_latency[SSV_GUARD_MAX_CANDIDATES];
} ssv_guard_state;

void ssv_guard_default_config(ssv_guard_config* cfg);
/* expected [n] (host), valid [n] (host, or NULL = all valid), 1 <= n <= SSV_GUARD_MAX_CANDIDATES.  SSV_EINVAL if no
 * candidate is valid or a parameter is out of range. */
int ssv_guard_init(ssv_guard_state* state, const ssv_guard_config* cfg, const double* expected, const uint8_t* valid,
                   int32_t n);
/* Feeds one verification step; returns the index (>= 0) of the strategy to use for the next step, or SSV_EINVAL. */
int ssv_guard_observe(ssv_guard_state* state, double accepted_tokens, double step_latency);

/*
 * Draft-tree flattening (Section 4.1; host only): reorders a tree given as parent indices (parents[i] in
 * {-1, 0..i-1}, -1 = child of the last committed token) into the verifier batch, breadth-first (siblings become
 * adjacent) or depth-first pre-order (parent and children become adjacent); children keep their relative order.
 * perm [n] (host, out): perm[new] = old index; new_parents [n] (host, out): parents in the new numbering, ready to
 * be uploaded as tree_parents of ssv_nsa_verify (q, gates and the draft K/V rows must be permuted with perm).
 * Returns SSV_OK, or SSV_EINVAL for a malformed tree.
 */
#define SSV_TREE_BFS 0
#define SSV_TREE_DFS 1
int ssv_tree_flatten(const int32_t* parents, int32_t n, int32_t order, int32_t* perm, int32_t* new_parents);

/* Validates p (host only, no GPU needed) and describes the launch plan.  Returns SSV_OK or an error code; a p that
 * this call accepts is accepted by ssv_nsa_workspace_bytes and ssv_nsa_verify too (the same checks run in all three). */
int ssv_nsa_plan_query(const ssv_nsa_params* p, ssv_nsa_plan* plan);

/* Scratch bytes ssv_nsa_verify needs for p; 0 if p is invalid. */
size_t ssv_nsa_workspace_bytes(const ssv_nsa_params* p);

/* 1 if this build has kernels for (dtype, d_k, d_v), else 0. */
int ssv_nsa_supported(int32_t dtype, int32_t d_k, int32_t d_v);

const char* ssv_nsa_strerror(int code);
const char* ssv_nsa_kernel_name(int kernel_index);
int ssv_nsa_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SSV_NSA_H */
