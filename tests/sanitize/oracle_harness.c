/*
 * TEST INFRASTRUCTURE -- runs the fp64 oracle (compiled together with this file under
 * -fsanitize=address,undefined) on a batch read from a flat binary file and writes its results.
 *
 * File layout (native endianness): int32 header[20] = {B, T, H, H_kv, d_k, d_v, l, d, l_sel, n_sel, w, n_init,
 * n_local, dtype, reuse, has_parents, S_cap, NC_cap, NS_cap, 0}, then q, k, v, k_cmp, v_cmp (element size 4 or
 * 2 by dtype), gates (float), seq_lens, n_cmp, n_query (int32 [B]), parents (int32 [B,T], if has_parents),
 * sel_idx (int32 [B,T,H_kv,n_sel]).  Output file: out (double [B,T,H,d_v]), sel_idx (int32), gap (double
 * [B,T,H_kv]), imp (double [B,T,H_kv,NS_cap]).
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

typedef struct {
    int32_t B, T, H, H_kv, d_k, d_v;
    int32_t l, d, l_sel, n_sel, w, n_init, n_local;
    int32_t dtype, reuse, n_threads;
    int64_t S_cap, NC_cap, NS_cap;
    double scale;
} ssv_oracle_params;

int ssv_oracle_nsa_verify(const ssv_oracle_params *p, const void *q, const void *k, const void *v,
                          const void *k_cmp, const void *v_cmp, const float *gates, const int32_t *seq_lens,
                          const int32_t *n_cmp, const int32_t *n_query, const int32_t *parents,
                          int32_t *sel_idx, double *out, double *gap, double *o_cmp_out, double *o_slc_out,
                          double *o_win_out, double *imp_out, double *p_cmp_out, const uint8_t *query_mask);

static void *slurp(FILE *f, size_t bytes)
{
    void *p = malloc(bytes ? bytes : 1);
    if (!p || fread(p, 1, bytes, f) != bytes) { fprintf(stderr, "short input\n"); exit(3); }
    return p;
}

int main(int argc, char **argv)
{
    if (argc != 3) return 2;
    FILE *f = fopen(argv[1], "rb");
    if (!f) return 2;
    int32_t h[20];
    if (fread(h, sizeof(int32_t), 20, f) != 20) return 3;
    ssv_oracle_params p = {h[0], h[1], h[2], h[3], h[4], h[5], h[6], h[7], h[8], h[9], h[10], h[11], h[12],
                           h[13], h[14], 1, h[16], h[17], h[18], 0.0};
    const size_t es = p.dtype ? 2 : 4;
    const size_t rows = (size_t)p.B * p.T * p.H, kv = (size_t)p.B * p.H_kv;
    void *q = slurp(f, rows * p.d_k * es);
    void *k = slurp(f, kv * p.S_cap * p.d_k * es);
    void *v = slurp(f, kv * p.S_cap * p.d_v * es);
    void *kc = slurp(f, kv * p.NC_cap * p.d_k * es);
    void *vc = slurp(f, kv * p.NC_cap * p.d_v * es);
    float *gates = slurp(f, rows * 3 * sizeof(float));
    int32_t *seq = slurp(f, (size_t)p.B * 4), *ncmp = slurp(f, (size_t)p.B * 4), *nq = slurp(f, (size_t)p.B * 4);
    int32_t *par = h[15] ? slurp(f, (size_t)p.B * p.T * 4) : NULL;
    const size_t n_idx = (size_t)p.B * p.T * p.H_kv * p.n_sel;
    int32_t *sel = slurp(f, n_idx * 4);
    fclose(f);
    double *out = calloc(rows * p.d_v, sizeof(double));
    double *gap = calloc((size_t)p.B * p.T * p.H_kv, sizeof(double));
    double *imp = calloc((size_t)p.B * p.T * p.H_kv * p.NS_cap, sizeof(double));
    const int rc = ssv_oracle_nsa_verify(&p, q, k, v, kc, vc, gates, seq, ncmp, nq, par, sel, out, gap, NULL, NULL,
                                         NULL, imp, NULL, NULL);
    if (rc != 0) return 4;
    FILE *o = fopen(argv[2], "wb");
    if (!o) return 2;
    fwrite(out, sizeof(double), rows * p.d_v, o);
    fwrite(sel, 4, n_idx, o);
    fwrite(gap, sizeof(double), (size_t)p.B * p.T * p.H_kv, o);
    fwrite(imp, sizeof(double), (size_t)p.B * p.T * p.H_kv * p.NS_cap, o);
    fclose(o);
    free(q); free(k); free(v); free(kc); free(vc); free(gates); free(seq); free(ncmp); free(nq); free(par);
    free(sel); free(out); free(gap); free(imp);
    return 0;
}
