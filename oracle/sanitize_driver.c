/*
 * TEST INFRASTRUCTURE ONLY: runs every entry point of ulorl_oracle.c once, in a build with
 * -fsanitize=address,undefined, on inputs read from a directory, and writes the results back
 * (tests/test_oracle_sanitized.py builds it, feeds it edge-case inputs, and compares the results
 * with those of the regular oracle library).  Every buffer is allocated with exactly the size the
 * oracle's contract states, so an access one element beyond it aborts the run.
 *
 * Files (little-endian, raw): meta.txt (one line of numbers, see main), logits.bin, y.i32,
 * cu.i32, seg.i32, old.f64, adv.f64, rows.i64, rewards.f64, trunc.u8, prev.i32, new.i32, eos.u8.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int ulorl_oracle_row_stats(const void *, int, int64_t, int64_t, int64_t, const int32_t *, double *, double *, double *);
int ulorl_oracle_token_terms(int64_t, const double *, const double *, const int32_t *, int32_t, const int32_t *, int32_t,
                             const double *, const double *, double, double, double, double, int, int, double, double *,
                             double *, uint8_t *, int32_t *, uint8_t *, double *, double *, double *, int64_t *);
int ulorl_oracle_dlogits(const void *, int, int64_t, int64_t, const int32_t *, const double *, const double *, double,
                         const int64_t *, int64_t, double *);
int ulorl_oracle_advantages(int32_t, int32_t, const double *, const uint8_t *, const int32_t *, int64_t, double, int,
                            double *, uint8_t *, double *, int64_t *);
int ulorl_oracle_segment_diagnostics(int64_t, int32_t, const int32_t *, const double *, const double *, const double *,
                                     const double *, const uint8_t *, const double *, double, double, int64_t *, double *,
                                     double *, int64_t *, double *, double *, int64_t *, int64_t *);
int ulorl_oracle_pool_step(int32_t, const int32_t *, const int32_t *, const uint8_t *, int32_t, int32_t, uint8_t *,
                           int32_t *, int32_t *, int32_t *, int32_t *, int64_t *, uint8_t *, int64_t *);

static char path[4096];
static const char *dir;

static void *slurp(const char *name, size_t bytes)
{
    snprintf(path, sizeof path, "%s/%s", dir, name);
    FILE *f = fopen(path, "rb");
    if (!f) { fprintf(stderr, "cannot open %s\n", path); exit(2); }
    void *p = malloc(bytes ? bytes : 1);
    if (fread(p, 1, bytes, f) != bytes) { fprintf(stderr, "short read %s\n", path); exit(2); }
    fclose(f);
    return p;
}

static void dump(const char *name, const void *p, size_t bytes)
{
    snprintf(path, sizeof path, "%s/%s", dir, name);
    FILE *f = fopen(path, "wb");
    if (!f || fwrite(p, 1, bytes, f) != bytes) { fprintf(stderr, "cannot write %s\n", path); exit(2); }
    fclose(f);
}

int main(int argc, char **argv)
{
    if (argc != 2) return 2;
    dir = argv[1];
    snprintf(path, sizeof path, "%s/meta.txt", dir);
    FILE *m = fopen(path, "r");
    if (!m) return 2;
    long long N, V, stride, R, K, seg_len, n_rows_sel, G, B, pool_seg, pool_max;
    int storage, is_mode, gate_mode, use_seg, use_old;
    double eps_low, eps_high, tau, sigma, denom, grad_out;
    if (fscanf(m, "%lld %lld %lld %d %lld %lld %lld %d %d %d %d %lf %lf %lf %lf %lf %lf %lld %lld %lld %lld %lld", &N, &V,
               &stride, &storage, &R, &K, &seg_len, &is_mode, &gate_mode, &use_seg, &use_old, &eps_low, &eps_high, &tau,
               &sigma, &denom, &grad_out, &n_rows_sel, &G, &B, &pool_seg, &pool_max) != 22)
        return 2;
    fclose(m);
    const size_t esz = storage == 0 ? 4 : storage == 1 ? 2 : 8;
    /* the last row is allocated up to V, not up to the stride: nothing beyond z[N-1, V-1] may be read */
    void *logits = slurp("logits.bin", (size_t)(((N - 1) * stride + V) * esz));
    int32_t *y = slurp("y.i32", (size_t)N * 4);
    int32_t *cu = slurp("cu.i32", (size_t)(R + 1) * 4);
    int32_t *seg_in = use_seg ? slurp("seg.i32", (size_t)N * 4) : NULL;
    double *old = use_old ? slurp("old.f64", (size_t)N * 8) : NULL;
    double *adv = slurp("adv.f64", (size_t)N * 8);
    int64_t *rows = slurp("rows.i64", (size_t)n_rows_sel * 8);

    double *lse = malloc((size_t)N * 8), *logp = malloc((size_t)N * 8), *ent = malloc((size_t)N * 8);
    int rc = ulorl_oracle_row_stats(logits, storage, N, V, stride, y, lse, logp, ent);
    dump("out_lse.f64", lse, (size_t)N * 8);
    dump("out_logp.f64", logp, (size_t)N * 8);
    dump("out_ent.f64", ent, (size_t)N * 8);
    if (rc != 0) { fprintf(stderr, "row_stats rc=%d\n", rc); return 3; }

    double loss = 0.0;
    double *hbar = malloc((size_t)R * 8), *ratio = malloc((size_t)N * 8), *sur = malloc((size_t)N * 8),
           *g = malloc((size_t)N * 8);
    uint8_t *gate = malloc((size_t)R), *mask = malloc((size_t)N);
    int32_t *seg = malloc((size_t)N * 4);
    int64_t cnt[3] = {0, 0, 0};
    rc = ulorl_oracle_token_terms(N, logp, ent, cu, (int32_t)R, seg_in, (int32_t)seg_len, old, adv, eps_low, eps_high, tau,
                                  sigma, is_mode, gate_mode, denom, &loss, hbar, gate, seg, mask, ratio, sur, g, cnt);
    if (rc != 0) { fprintf(stderr, "token_terms rc=%d\n", rc); return 3; }
    dump("out_loss.f64", &loss, 8);
    dump("out_hbar.f64", hbar, (size_t)R * 8);
    dump("out_gate.u8", gate, (size_t)R);
    dump("out_seg.i32", seg, (size_t)N * 4);
    dump("out_mask.u8", mask, (size_t)N);
    dump("out_ratio.f64", ratio, (size_t)N * 8);
    dump("out_sur.f64", sur, (size_t)N * 8);
    dump("out_g.f64", g, (size_t)N * 8);
    dump("out_cnt.i64", cnt, 24);

    double *dz = malloc((size_t)n_rows_sel * (size_t)V * 8);
    ulorl_oracle_dlogits(logits, storage, V, stride, y, lse, g, grad_out, rows, n_rows_sel, dz);
    dump("out_dz.f64", dz, (size_t)n_rows_sel * (size_t)V * 8);

    int64_t *d_count = malloc((size_t)K * 8), *d_clip = malloc((size_t)K * 8), *d_mask = malloc((size_t)K * 8), oor = 0;
    double *d_rs = malloc((size_t)K * 8), *d_rm = malloc((size_t)K * 8), *d_kl = malloc((size_t)K * 8),
           *d_en = malloc((size_t)K * 8);
    ulorl_oracle_segment_diagnostics(N, (int32_t)K, seg, ratio, logp, old, ent, mask, adv, eps_low, eps_high, d_count, d_rs,
                                     d_rm, d_clip, d_kl, d_en, d_mask, &oor);
    dump("out_d_count.i64", d_count, (size_t)K * 8);
    dump("out_d_rs.f64", d_rs, (size_t)K * 8);
    dump("out_d_rm.f64", d_rm, (size_t)K * 8);
    dump("out_d_clip.i64", d_clip, (size_t)K * 8);
    dump("out_d_kl.f64", d_kl, (size_t)K * 8);
    dump("out_d_en.f64", d_en, (size_t)K * 8);
    dump("out_d_mask.i64", d_mask, (size_t)K * 8);
    dump("out_d_oor.i64", &oor, 8);

    double *rewards = slurp("rewards.f64", (size_t)R * 8);
    uint8_t *trunc = slurp("trunc.u8", (size_t)R);
    double *resp_adv = malloc((size_t)R * 8), *tok_adv = malloc((size_t)N * 8);
    uint8_t *keep = malloc((size_t)(R / G));
    int64_t kept = 0;
    rc = ulorl_oracle_advantages((int32_t)R, (int32_t)G, rewards, trunc, cu, N, 1e-6, 0, resp_adv, keep, tok_adv, &kept);
    if (rc != 0) { fprintf(stderr, "advantages rc=%d\n", rc); return 3; }
    dump("out_resp_adv.f64", resp_adv, (size_t)R * 8);
    dump("out_keep.u8", keep, (size_t)(R / G));
    dump("out_tok_adv.f64", tok_adv, (size_t)N * 8);
    dump("out_kept.i64", &kept, 8);

    int32_t *prev = slurp("prev.i32", (size_t)B * 4), *newl = slurp("new.i32", (size_t)B * 4);
    uint8_t *eos = slurp("eos.u8", (size_t)B);
    uint8_t *state = malloc((size_t)B), *ptrunc = malloc((size_t)B);
    int32_t *total = malloc((size_t)B * 4), *segs = malloc((size_t)B * 4), *unf = malloc((size_t)B * 4),
            *expi = malloc((size_t)B * 4);
    int64_t *pcu = malloc((size_t)(B + 1) * 8), counts[5];
    rc = ulorl_oracle_pool_step((int32_t)B, prev, newl, eos, (int32_t)pool_seg, (int32_t)pool_max, state, total, segs, unf,
                                expi, pcu, ptrunc, counts);
    if (rc != 0) { fprintf(stderr, "pool_step rc=%d\n", rc); return 3; }
    dump("out_state.u8", state, (size_t)B);
    dump("out_total.i32", total, (size_t)B * 4);
    dump("out_segs.i32", segs, (size_t)B * 4);
    dump("out_unf.i32", unf, (size_t)counts[0] * 4);
    dump("out_exp.i32", expi, (size_t)counts[1] * 4);
    dump("out_pcu.i64", pcu, (size_t)(counts[1] + 1) * 8);
    dump("out_ptrunc.u8", ptrunc, (size_t)counts[1]);
    dump("out_counts.i64", counts, 40);

    free(logits); free(y); free(cu); free(seg_in); free(old); free(adv); free(rows); free(lse); free(logp); free(ent);
    free(hbar); free(ratio); free(sur); free(g); free(gate); free(mask); free(seg); free(dz);
    free(d_count); free(d_clip); free(d_mask); free(d_rs); free(d_rm); free(d_kl); free(d_en);
    free(rewards); free(trunc); free(resp_adv); free(tok_adv); free(keep);
    free(prev); free(newl); free(eos); free(state); free(ptrunc); free(total); free(segs); free(unf); free(expi); free(pcu);
    printf("sanitized oracle run complete\n");
    return 0;
}
