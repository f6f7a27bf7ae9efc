/* Driver for the sanitizer build of the CPU oracle (test infrastructure): reads a model blob and
 * inputs written by tests/test_oracle_sanitize.py, runs every entry point of oracle/hawk_oracle.h
 * once or more, prints the tokens.  Built with -fsanitize=address,undefined, so any out-of-bounds
 * access, use after free, signed overflow or misaligned access in the oracle ends the run. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "../oracle/hawk_oracle.h"

#define CHECK(x) do { int rc_ = (x); if (rc_ != 0) { fprintf(stderr, "FAILED %s -> %d (line %d)\n", #x, rc_, __LINE__); return 2; } } while (0)

static void* slurp(FILE* f, size_t n) {
    void* p = malloc(n ? n : 1);
    if (!p || fread(p, 1, n, f) != n) { fprintf(stderr, "short read\n"); exit(3); }
    return p;
}

int main(int argc, char** argv) {
    if (argc != 2) return 1;
    FILE* f = fopen(argv[1], "rb");
    if (!f) return 1;
    int32_t hdr[16];
    float fl[4];
    int64_t blob_bytes;
    if (fread(hdr, 4, 16, f) != 16 || fread(fl, 4, 4, f) != 4 || fread(&blob_bytes, 8, 1, f) != 1) return 1;
    const int samp_lo = hdr[0], samp_n = hdr[1], batch = hdr[2], use_cfg = hdr[3], n_cond = hdr[4], gh = hdr[5], gw = hdr[6];
    const int k_max = hdr[7], k = hdr[8], top_k = hdr[9], d = hdr[10], seed = hdr[11], vs = hdr[12];
    const float temperature = fl[0], cfg_scale = fl[1];
    void* blob = slurp(f, (size_t)blob_bytes);
    float* cond = slurp(f, (size_t)batch * n_cond * d * 4);
    float* uncond = use_cfg ? slurp(f, (size_t)batch * n_cond * d * 4) : NULL;
    fclose(f);
    const int N = gh * gw, S = batch * (use_cfg ? 2 : 1);

    orc_model* m = orc_load(blob, (size_t)blob_bytes, samp_lo, samp_n, fl[2], fl[3]);
    if (!m) return 4;
    /* 1. the generation loop */
    orc_state* s = orc_new_state(m, batch, use_cfg, n_cond, gh, gw, k_max);
    if (!s) return 4;
    int32_t* grid = calloc((size_t)batch * N, 4);
    int64_t stats[4];
    CHECK(orc_generate(s, cond, uncond, n_cond, k, temperature, top_k, cfg_scale, (uint64_t)seed, grid, stats));
    printf("grid");
    for (int i = 0; i < batch * N; ++i) printf(" %d", grid[i]);
    printf("\nstats %lld %lld %lld %lld\n", (long long)stats[0], (long long)stats[1], (long long)stats[2], (long long)stats[3]);
    orc_free_state(s);

    /* 2. the calls one by one, with read-backs, a forced draft, a re-synchronisation and steps up to the
     * end of the image (where fewer than k positions are left) */
    s = orc_new_state(m, batch, use_cfg, n_cond, gh, gw, k_max);
    if (!s) return 4;
    float* u = malloc((size_t)batch * (k_max + 1) * 4);
    int32_t* dr = malloc((size_t)batch * (k_max + 1) * 4);
    int32_t* na = malloc((size_t)batch * 4);
    int32_t* tk = malloc((size_t)batch * (k_max + 1) * 4);
    int32_t* nn = malloc((size_t)batch * 4);
    float* lg = malloc((size_t)batch * (k_max + 1) * vs * 4);
    double* hp = malloc((size_t)S * d * 8);
    for (int i = 0; i < batch * (k_max + 1); ++i) u[i] = (float)((i * 37 + 11) % 97) / 97.0f;
    CHECK(orc_prefill(s, cond, uncond, n_cond, temperature, top_k, cfg_scale, u));
    int step = 0;
    for (;;) {
        CHECK(orc_get_n(s, nn));
        int done = 1;
        for (int b = 0; b < batch; ++b) done = done && nn[b] >= N;
        if (done) break;
        const int kk = step % (k_max + 1);
        if (step % 3 == 2 && kk > 0) {
            for (int i = 0; i < batch * kk; ++i) dr[i] = samp_lo + (i * 5 + step) % vs;
            CHECK(orc_draft_forced(s, kk, dr, step % 2));
        } else {
            CHECK(orc_draft(s, kk, kk ? u : NULL, kk ? dr : NULL));
        }
        if (kk) CHECK(orc_get_draft_logits(s, lg));
        CHECK(orc_verify(s, kk, kk ? u + 1 : NULL, u + 2, na, tk));
        CHECK(orc_get_logits(s, lg));
        CHECK(orc_get_hprev(s, hp));
        printf("step %d k %d:", step, kk);
        for (int b = 0; b < batch; ++b) printf(" a=%d t0=%d", na[b], tk[b * (kk + 1)]);
        printf("\n");
        ++step;
    }
    CHECK(orc_get_grid(s, grid));
    /* rewind two tokens and feed them again */
    for (int b = 0; b < batch; ++b) { nn[b] = N - 2; tk[b * 2] = grid[b * N + N - 2]; tk[b * 2 + 1] = grid[b * N + N - 1]; }
    CHECK(orc_force(s, nn, tk, 2));
    /* one target row and one head evaluation on their own */
    double* x = calloc((size_t)d, 8);
    double* g = calloc((size_t)d, 8);
    x[0] = 1.0;
    CHECK(orc_forward_row(s, 0, n_cond + N - 1, x, lg));
    CHECK(orc_draft_head(s, x, samp_lo, -1, g, lg));
    orc_free_state(s);

    /* 3. the context-free routines on synthetic rows */
    {
        const int n = 37, mm = 3;
        float p[37], q[3 * 37], p4[4 * 37], ua[3] = {0.9f, 0.99f, 0.5f};
        int32_t cand[3] = {4, 36, 0}, tok = -1, toks[4];
        double resid[3], w[37];
        for (int i = 0; i < n; ++i) p[i] = (float)((i * 7) % 11) * 0.3f;
        for (int i = 0; i < mm * n; ++i) q[i] = (float)((i * 5) % 13) * 0.25f;
        int a = orc_multi_verify(mm, n, p, q, cand, 1.0f, 9, ua, 0.3f, &tok, resid);
        printf("multi %d %d\n", a, tok);
        for (int i = 0; i < 4 * n; ++i) p4[i] = i < mm * n ? q[i] : p[i - mm * n];   /* k + 1 target rows, the first k == q */
        a = orc_spec_sample(3, n, p4, q, cand, 0, 1.0f, n, ua, 0.7f, toks);      /* p == q: everything accepted */
        printf("spec %d %d\n", a, toks[3]);
        const double z = orc_warp(p, n, 0.7f, 5, w);
        printf("draw %d %d\n", orc_inv_cdf(w, n, z, 0.0f), orc_inv_cdf(w, n, z, 0.99999994f));
        orc_guide(p, q, 3.0f, n, q + n);
        double mg[3];
        orc_margins(mg, 1);
    }
    free(x); free(g); free(u); free(dr); free(na); free(tk); free(nn); free(lg); free(hp); free(grid);
    orc_free_model(m);
    free(blob); free(cond); free(uncond);
    printf("threads %d\nOK\n", orc_num_threads());
    return 0;
}
