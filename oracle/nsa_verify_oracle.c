/*
 * TEST INFRASTRUCTURE -- CPU oracle for NSA speculative verification attention.
 *
 * A plain, slow, double-precision implementation of what the verification path
 * computes, written out per verifier query exactly as the definition reads: the
 * paper's exact merged-schedule execution is stated to be equivalent to running every
 * verifier query on its own (Section 4.2), so the oracle IS that per-query definition
 * of the three NSA branches (Section 2.2: compression, selection, sliding window, fused
 * by gates) under the draft-tree mask (Section 2.1, Section 4.1).  There is no tiling,
 * no fusion, no sharing of loads between queries and no reduced precision here.
 *
 * It shares no code with the HIP library and is never called by the product path: only
 * the tests, the smoke check and the benchmark's cpu_baseline leg load it.
 *
 * Notation (Section 2.2 and Section 7 setup): compression blocks of length l and stride
 * d, selection blocks of size l' (l_sel), n selected blocks per query (n_sel), window w.
 * Per sequence b: L committed tokens in slots 0..L-1, draft token i in slot L+i;
 * parents[i] in {-1, 0..i-1}, -1 meaning "child of the last committed token".
 *
 * Steps for sequence b, verifier query i, KV group g (heads h with h / H_g == g):
 *  O0  visibility: slot s is visible iff s < L, or s-L is i itself or an ancestor of i.
 *      kpos(s) = s for s < L, L + depth(s-L) otherwise;  pos(i) = L + depth(i).
 *      E(i) = L + (number of leading draft slots 0,1,2,... that are all visible).
 *  O1  compressed block c (slots [c*d, c*d+l)) is visible iff c < n_cmp[b] and
 *      c*d + l <= E(i): only complete blocks made of tokens the query may see.
 *  O2  s_c = scale * <q[i,h], k_cmp[g,c]>;  p = softmax over visible c.
 *  O3  o_cmp = sum_c p_c v_cmp[g,c]   (zero when nothing is visible).
 *  O4  importance of selection block j for the group:
 *      imp[j] = sum_{h in g} sum_{m < l'/d} sum_{n' < l/d} p_h[(l'/d) j + m - n'],
 *      out-of-range or invisible indices contributing zero: every stride-d chunk of
 *      block j collects the probability of each compression block that covers it.
 *  O5  J = floor((L+i) / l') (block of the query's own slot); candidates 0..J.
 *      Forced: blocks 0..n_init-1 and J-n_local+1..J (clipped, de-duplicated).
 *      n_eff = min(n_sel, J+1).  Chosen = forced + the n_eff-|forced| remaining
 *      candidates of largest imp, ties to the smaller index.  Written ascending, -1 padded.
 *      gap = (smallest chosen free imp) - (largest unchosen imp), +inf if either is absent.
 *  O6  o_slc = softmax attention over visible slots whose block floor(s/l') is chosen.
 *  O7  o_win = softmax attention over visible slots with pos(i)-w < kpos(s) <= pos(i).
 *  O8  out = g_cmp o_cmp + g_slc o_slc + g_win o_win.
 *  O9  reuse mode (Section 5.2): the chosen set is read from sel_idx (negative, repeated
 *      and out-of-range entries ignored); O4-O5 are skipped; everything else is the same.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    int32_t B, T, H, H_kv, d_k, d_v;
    int32_t l, d, l_sel, n_sel, w, n_init, n_local;
    int32_t dtype;  /* 0: float32 arrays, 1: bfloat16 bit patterns (uint16) */
    int32_t reuse;  /* 0: compute sel_idx, 1: sel_idx is an input */
    int32_t n_threads; /* 0: OpenMP default */
    int64_t S_cap, NC_cap, NS_cap; /* slots per head in k/v, rows per head in k_cmp/v_cmp, columns of imp */
    double scale;   /* <= 0: 1/sqrt(d_k) */
} ssv_oracle_params;

static inline double ld(const void *base, int dtype, int64_t idx)
{
    if (dtype == 0)
        return (double)((const float *)base)[idx];
    uint32_t bits = ((uint32_t)((const uint16_t *)base)[idx]) << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

/* softmax attention of one query row over the listed rows of (kmat, vmat) */
static void attend(const void *q, int64_t q_off, const void *kmat, int64_t k_off, int64_t k_stride,
                   const void *vmat, int64_t v_off, int64_t v_stride, const int64_t *rows, int64_t n_rows,
                   int d_k, int d_v, int dtype, double scale, double *score_tmp, double *prob_out, double *o)
{
    for (int e = 0; e < d_v; ++e) o[e] = 0.0;
    if (n_rows == 0) return;
    double mx = -INFINITY;
    for (int64_t r = 0; r < n_rows; ++r) {
        double acc = 0.0;
        for (int e = 0; e < d_k; ++e)
            acc += ld(q, dtype, q_off + e) * ld(kmat, dtype, k_off + rows[r] * k_stride + e);
        score_tmp[r] = scale * acc;
        if (score_tmp[r] > mx) mx = score_tmp[r];
    }
    double z = 0.0;
    for (int64_t r = 0; r < n_rows; ++r) {
        score_tmp[r] = exp(score_tmp[r] - mx);
        z += score_tmp[r];
    }
    for (int64_t r = 0; r < n_rows; ++r) {
        double pr = score_tmp[r] / z;
        if (prob_out) prob_out[r] = pr;
        for (int e = 0; e < d_v; ++e)
            o[e] += pr * ld(vmat, dtype, v_off + rows[r] * v_stride + e);
    }
}

#ifdef _OPENMP
#include <omp.h>
#endif

int ssv_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * Arrays (C order): q [B,T,H,d_k]; k [B,H_kv,S_cap,d_k]; v [B,H_kv,S_cap,d_v];
 * k_cmp [B,H_kv,NC_cap,d_k]; v_cmp [B,H_kv,NC_cap,d_v]; gates [B,T,H,3] (cmp, slc, win);
 * seq_lens, n_cmp, n_query [B]; parents [B,T] or NULL (linear chain);
 * sel_idx [B,T,H_kv,n_sel]; out, o_cmp, o_slc, o_win [B,T,H,d_v] doubles (branch outputs optional);
 * gap [B,T,H_kv] optional; imp [B,T,H_kv,NS_cap] optional; p_cmp [B,T,H,NC_cap] optional;
 * query_mask [B,T] optional: when given, only queries with a non-zero entry are computed.
 * Rows of queries i >= n_query[b] are left untouched.  Returns 0, or -1 on a bad argument.
 */
int ssv_oracle_nsa_verify(const ssv_oracle_params *p, const void *q, const void *k, const void *v,
                          const void *k_cmp, const void *v_cmp, const float *gates, const int32_t *seq_lens,
                          const int32_t *n_cmp, const int32_t *n_query, const int32_t *parents,
                          int32_t *sel_idx, double *out, double *gap, double *o_cmp_out, double *o_slc_out,
                          double *o_win_out, double *imp_out, double *p_cmp_out, const uint8_t *query_mask)
{
    if (!p || !q || !k || !v || !k_cmp || !v_cmp || !gates || !seq_lens || !n_cmp || !sel_idx || !out) return -1;
    const int B = p->B, T = p->T, H = p->H, H_kv = p->H_kv, d_k = p->d_k, d_v = p->d_v;
    if (B < 1 || T < 1 || H_kv < 1 || H % H_kv || p->l < 1 || p->d < 1 || p->l_sel < 1) return -1;
    if (p->l % p->d || p->l_sel % p->d || p->n_sel < p->n_init + p->n_local) return -1;
    const int H_g = H / H_kv, dtype = p->dtype;
    const int a_ratio = p->l_sel / p->d, b_ratio = p->l / p->d;
    const double scale = p->scale > 0 ? p->scale : 1.0 / sqrt((double)d_k);
    int status = 0;

#ifdef _OPENMP
    if (p->n_threads > 0) omp_set_num_threads(p->n_threads);
#endif
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t unit = 0; unit < (int64_t)B * T * H_kv; ++unit) {
        const int b = (int)(unit / ((int64_t)T * H_kv));
        const int i = (int)((unit / H_kv) % T);
        const int g = (int)(unit % H_kv);
        const int Tq = n_query ? n_query[b] : T;
        if (i >= Tq) continue;
        if (query_mask && !query_mask[(int64_t)b * T + i]) continue;
        const int64_t L = seq_lens[b];

        /* O0: ancestry, depths, contiguous visible extent */
        int *depth = (int *)malloc(sizeof(int) * T);
        unsigned char *is_anc = (unsigned char *)calloc(T, 1);
        for (int t = 0; t < Tq; ++t) {
            int par = parents ? parents[(int64_t)b * T + t] : t - 1;
            depth[t] = par < 0 ? 0 : depth[par] + 1;
        }
        for (int t = i; t >= 0; t = parents ? parents[(int64_t)b * T + t] : t - 1) is_anc[t] = 1;
        const int64_t pos_i = L + depth[i];
        int lead = 0;
        while (lead < Tq && is_anc[lead]) ++lead;
        const int64_t E = L + lead;
        const int64_t n_slots = L + Tq;

        /* O1: visible compressed blocks */
        int64_t ncv = 0;
        int64_t *cmp_rows = (int64_t *)malloc(sizeof(int64_t) * (n_cmp[b] > 0 ? n_cmp[b] : 1));
        for (int64_t c = 0; c < n_cmp[b]; ++c)
            if (c * p->d + p->l <= E) cmp_rows[ncv++] = c;

        const int64_t J = (L + i) / p->l_sel;
        double *imp = (double *)calloc(J + 1, sizeof(double));
        double *tmp = (double *)malloc(sizeof(double) * (n_slots > ncv ? n_slots : ncv + 1));
        double *prob = (double *)malloc(sizeof(double) * (ncv + 1));
        double *ocmp = (double *)malloc(sizeof(double) * d_v * H_g);

        /* O2-O4 */
        for (int hh = 0; hh < H_g; ++hh) {
            const int h = g * H_g + hh;
            const int64_t q_off = (((int64_t)b * T + i) * H + h) * d_k;
            const int64_t kc_off = ((int64_t)b * H_kv + g) * p->NC_cap * d_k;
            const int64_t vc_off = ((int64_t)b * H_kv + g) * p->NC_cap * d_v;
            attend(q, q_off, k_cmp, kc_off, d_k, v_cmp, vc_off, d_v, cmp_rows, ncv, d_k, d_v, dtype, scale,
                   tmp, prob, ocmp + (int64_t)hh * d_v);
            if (p_cmp_out) {
                double *dst = p_cmp_out + (((int64_t)b * T + i) * H + h) * p->NC_cap;
                for (int64_t c = 0; c < p->NC_cap; ++c) dst[c] = 0.0;
                for (int64_t r = 0; r < ncv; ++r) dst[cmp_rows[r]] = prob[r];
            }
            /* visible blocks are 0..ncv-1 in order (visibility is a prefix), so prob[c] is block c */
            for (int64_t j = 0; j <= J; ++j)
                for (int m = 0; m < a_ratio; ++m)
                    for (int n2 = 0; n2 < b_ratio; ++n2) {
                        int64_t c = (int64_t)a_ratio * j + m - n2;
                        if (c >= 0 && c < ncv) imp[j] += prob[c];
                    }
        }
        if (imp_out) {
            double *dst = imp_out + (((int64_t)b * T + i) * H_kv + g) * p->NS_cap;
            for (int64_t j = 0; j < p->NS_cap; ++j) dst[j] = j <= J ? imp[j] : 0.0;
        }

        /* O5 / O9: chosen set */
        const int64_t n_blk = (n_slots + p->l_sel - 1) / p->l_sel;
        unsigned char *chosen = (unsigned char *)calloc(n_blk > J + 1 ? n_blk : J + 1, 1);
        int32_t *sel = sel_idx + (((int64_t)b * T + i) * H_kv + g) * p->n_sel;
        if (p->reuse) {
            for (int e = 0; e < p->n_sel; ++e)
                if (sel[e] >= 0 && sel[e] < n_blk) chosen[sel[e]] = 1;
        } else {
            unsigned char *forced = (unsigned char *)calloc(J + 1, 1);
            int n_forced = 0;
            for (int64_t j = 0; j < p->n_init && j <= J; ++j)
                if (!forced[j]) { forced[j] = 1; ++n_forced; }
            for (int64_t j = J - p->n_local + 1; j <= J; ++j)
                if (j >= 0 && !forced[j]) { forced[j] = 1; ++n_forced; }
            const int64_t n_eff = p->n_sel < J + 1 ? p->n_sel : J + 1;
            for (int64_t j = 0; j <= J; ++j) chosen[j] = forced[j];
            double min_chosen = INFINITY;
            for (int64_t pick = n_forced; pick < n_eff; ++pick) {
                int64_t best = -1;
                for (int64_t j = 0; j <= J; ++j)
                    if (!chosen[j] && (best < 0 || imp[j] > imp[best])) best = j; /* strict >: ties keep the smaller j */
                chosen[best] = 1;
                if (imp[best] < min_chosen) min_chosen = imp[best];
            }
            double max_unchosen = -INFINITY;
            for (int64_t j = 0; j <= J; ++j)
                if (!chosen[j] && imp[j] > max_unchosen) max_unchosen = imp[j];
            if (gap)
                gap[((int64_t)b * T + i) * H_kv + g] =
                    (isinf(min_chosen) || isinf(max_unchosen)) ? INFINITY : min_chosen - max_unchosen;
            int e = 0;
            for (int64_t j = 0; j <= J; ++j)
                if (chosen[j]) sel[e++] = (int32_t)j;
            for (; e < p->n_sel; ++e) sel[e] = -1;
            free(forced);
        }

        /* O6-O7: member slots of the two raw-KV branches */
        int64_t *slc_rows = (int64_t *)malloc(sizeof(int64_t) * n_slots);
        int64_t *win_rows = (int64_t *)malloc(sizeof(int64_t) * n_slots);
        int64_t n_slc = 0, n_win = 0;
        for (int64_t s = 0; s < n_slots; ++s) {
            const int visible = s < L || is_anc[s - L];
            if (!visible) continue;
            const int64_t kpos = s < L ? s : L + depth[s - L];
            if (chosen[s / p->l_sel]) slc_rows[n_slc++] = s;
            if (kpos > pos_i - p->w && kpos <= pos_i) win_rows[n_win++] = s;
        }
        double *oslc = (double *)malloc(sizeof(double) * d_v);
        double *owin = (double *)malloc(sizeof(double) * d_v);
        for (int hh = 0; hh < H_g; ++hh) {
            const int h = g * H_g + hh;
            const int64_t row = ((int64_t)b * T + i) * H + h;
            const int64_t k_off = ((int64_t)b * H_kv + g) * p->S_cap * d_k;
            const int64_t v_off = ((int64_t)b * H_kv + g) * p->S_cap * d_v;
            attend(q, row * d_k, k, k_off, d_k, v, v_off, d_v, slc_rows, n_slc, d_k, d_v, dtype, scale, tmp, NULL, oslc);
            attend(q, row * d_k, k, k_off, d_k, v, v_off, d_v, win_rows, n_win, d_k, d_v, dtype, scale, tmp, NULL, owin);
            const float *gt = gates + row * 3;
            for (int e = 0; e < d_v; ++e) {
                const double oc = ocmp[(int64_t)hh * d_v + e];
                out[row * d_v + e] = (double)gt[0] * oc + (double)gt[1] * oslc[e] + (double)gt[2] * owin[e]; /* O8 */
                if (o_cmp_out) o_cmp_out[row * d_v + e] = oc;
                if (o_slc_out) o_slc_out[row * d_v + e] = oslc[e];
                if (o_win_out) o_win_out[row * d_v + e] = owin[e];
            }
        }
        free(oslc); free(owin); free(slc_rows); free(win_rows); free(chosen);
        free(ocmp); free(prob); free(tmp); free(imp); free(cmp_rows); free(is_anc); free(depth);
    }
    return status;
}
