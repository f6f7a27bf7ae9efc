/*
 * CPU oracle: see hawk_oracle.h for scope, citations and the list of pins.
 * TEST INFRASTRUCTURE ONLY - never part of the product path.
 *
 * Arithmetic: weights are used at their stored value (fp32, or bf16 widened exactly);
 * every activation, accumulator, cache entry and probability is fp64.  The only fp32
 * quantities are the ones the interface defines as fp32: per-stream logits, the guidance
 * combination of two logit rows, the temperature scaling, and the uniforms.
 */
#include "hawk_oracle.h"

#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif
#include <stdlib.h>
#include <string.h>

struct orc_model {
    int dtype, L, d, H, hd, m, V, samp_lo, Vs;
    double eps, theta;
    const uint8_t* blob;
    size_t esz;
    size_t off_E, off_gf, off_Wout, off_Wd;
    size_t *off_g1, *off_Wq, *off_Wk, *off_Wv, *off_Wo, *off_g2, *off_W1, *off_W3, *off_W2;
};

struct orc_state {
    const orc_model* M;
    int B, S, use_cfg, Cmax, C, gh, gw, N, kmax, Tmax;
    float temperature, cfg_scale;
    int top_k;
    int phase; /* 0 = created, 1 = prefilled (draft next), 2 = drafted (verify next) */
    int k_last, q_onehot;
    double *Kc, *Vc;  /* [S][L][Tmax][d] */
    int32_t* grid;    /* [B][N] */
    int32_t* n;       /* [B] committed image tokens */
    int32_t* k_eff;   /* [B] drafts of the current step, -1 = prompt finished */
    int32_t* draft;   /* [B][kmax] */
    double* h_prev;   /* [S][d] */
    double* hid;      /* [S][kmax+1][d] */
    float* lq;        /* [B][kmax][Vs] draft logits after guidance */
    float* lp;        /* [B][kmax+1][Vs] target logits after guidance */
};

/* ------------------------------------------------------------------ helpers */

static double g_margin[3] = {1e300, 1e300, 1e300};

void orc_margins(double out[3], int reset) {
    if (out) memcpy(out, g_margin, sizeof g_margin);
    if (reset) g_margin[0] = g_margin[1] = g_margin[2] = 1e300;
}

static inline float bf16_widen(uint16_t b) {
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

/* Value of element idx of the tensor that starts at byte offset off. */
static inline double wval(const orc_model* M, size_t off, size_t idx) {
    if (M->dtype == 0) return (double)((const float*)(M->blob + off))[idx];
    return (double)bf16_widen(((const uint16_t*)(M->blob + off))[idx]);
}

/* y[o] = sum_i W[o][i] * x[i], W row-major [rows][cols]. */
static void matvec(const orc_model* M, size_t off, int row0, int rows, int cols,
                   const double* x, double* y) {
#pragma omp parallel for schedule(static)
    for (int o = 0; o < rows; ++o) {
        size_t base = (size_t)(row0 + o) * (size_t)cols;
        double acc = 0.0;
        if (M->dtype == 0) {
            const float* w = (const float*)(M->blob + off) + base;
            for (int i = 0; i < cols; ++i) acc += (double)w[i] * x[i];
        } else {
            const uint16_t* w = (const uint16_t*)(M->blob + off) + base;
            for (int i = 0; i < cols; ++i) acc += (double)bf16_widen(w[i]) * x[i];
        }
        y[o] = acc;
    }
}

/* RMSNorm: out_i = x_i / sqrt(mean(x^2) + eps) * g_i. */
static void rmsnorm(const orc_model* M, size_t off_g, const double* x, double* out) {
    double ss = 0.0;
    for (int i = 0; i < M->d; ++i) ss += x[i] * x[i];
    double r = 1.0 / sqrt(ss / (double)M->d + M->eps);
    for (int i = 0; i < M->d; ++i) out[i] = x[i] * r * wval(M, off_g, (size_t)i);
}

/* Rotary embedding: pair (2j, 2j+1) of every head turned by pos * theta^(-2j/hd). */
static void rope(const orc_model* M, double* v, int pos) {
    for (int h = 0; h < M->H; ++h)
        for (int j = 0; j < M->hd / 2; ++j) {
            double ang = (double)pos * pow(M->theta, -2.0 * (double)j / (double)M->hd);
            double c = cos(ang), s = sin(ang);
            double* p = v + (size_t)h * M->hd + 2 * j;
            double a = p[0], b = p[1];
            p[0] = a * c - b * s;
            p[1] = a * s + b * c;
        }
}

static void embed(const orc_model* M, int tok, double* x) {
    for (int i = 0; i < M->d; ++i) x[i] = wval(M, M->off_E, (size_t)tok * M->d + i);
}

/* logits (fp32) of the sampled vocabulary slice from a hidden state before the final norm */
static void lm_head(const orc_model* M, const double* h, float* logits) {
    double* a = (double*)malloc(sizeof(double) * (size_t)M->d);
    double* y = (double*)malloc(sizeof(double) * (size_t)M->Vs);
    rmsnorm(M, M->off_gf, h, a);
    matvec(M, M->off_Wout, M->samp_lo, M->Vs, M->d, a, y);
    for (int j = 0; j < M->Vs; ++j) logits[j] = (float)y[j];
    free(a);
    free(y);
}

/* Classifier-free guidance on two fp32 logit rows: l_u + s * (l_c - l_u). */
static void guide(const float* lc, const float* lu, float s, int n, float* out) {
    for (int j = 0; j < n; ++j) out[j] = fmaf(s, lc[j] - lu[j], lu[j]);
}

void orc_guide(const float* lc, const float* lu, float scale, int n, float* out) { guide(lc, lu, scale, n, out); }

/* ------------------------------------------------------------ uniform source */

static inline uint64_t mix64(uint64_t z) {
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

/* Counter-based uniform in [0,1) with 24 random bits: two rounds of the splitmix64
 * finaliser over (seed, sequence, step, slot). */
float orc_uniform(uint64_t seed, uint32_t seq, uint32_t step, uint32_t slot) {
    uint64_t ctr = ((uint64_t)seq << 44) | ((uint64_t)step << 8) | (uint64_t)(slot & 0xFFu);
    uint64_t z = mix64(seed + 0x9E3779B97F4A7C15ull);
    z = mix64(z + 0x9E3779B97F4A7C15ull * (ctr + 1));
    return (float)(z >> 40) * (1.0f / 16777216.0f);
}

/* ------------------------------------------------------------ sampling stage */

typedef struct { float z; int idx; } zi_t;

static int cmp_zi(const void* a, const void* b) {
    const zi_t* x = (const zi_t*)a;
    const zi_t* y = (const zi_t*)b;
    if (x->z > y->z) return -1;
    if (x->z < y->z) return 1;
    return (x->idx > y->idx) - (x->idx < y->idx);
}

/* Temperature + top-k warp of one logit row into unnormalised weights w (fp64);
 * returns their sum.  temperature == 0 or top_k == 1: one-hot at the arg-max (lowest
 * index among equals).  Otherwise z = l * (1/T) in fp32, keep the top_k largest z
 * (equal values: lower index first), w = exp(z - z_max) on the kept entries. */
double orc_warp(const float* l, int n, float temperature, int top_k, double* w) {
    for (int j = 0; j < n; ++j) w[j] = 0.0;
    if (temperature == 0.0f || top_k == 1) {
        int best = 0;
        for (int j = 1; j < n; ++j)
            if (l[j] > l[best]) best = j;
        w[best] = 1.0;
        return 1.0;
    }
    float inv_t = 1.0f / temperature;
    zi_t* s = (zi_t*)malloc(sizeof(zi_t) * (size_t)n);
    for (int j = 0; j < n; ++j) {
        s[j].z = l[j] * inv_t;
        s[j].idx = j;
    }
    qsort(s, (size_t)n, sizeof(zi_t), cmp_zi);
    int K = top_k < n ? top_k : n;
    if (K < n) {
        double gap = (double)s[K - 1].z - (double)s[K].z;
        if (gap < g_margin[2]) g_margin[2] = gap;
    }
    double zmax = (double)s[0].z;
    for (int r = 0; r < K; ++r) w[s[r].idx] = exp((double)s[r].z - zmax);
    free(s);
    double total = 0.0;
    for (int j = 0; j < n; ++j) total += w[j];
    return total;
}

/* Inverse-CDF draw over ascending index: first j whose running sum exceeds u * total;
 * if rounding leaves none, the last index with positive weight. */
int orc_inv_cdf(const double* w, int n, double total, float u) {
    double target = (double)u * total, c = 0.0;
    int last = -1;
    for (int j = 0; j < n; ++j) {
        if (w[j] > 0.0) {
            double c_new = c + w[j];
            if (c_new > target) {
                double m1 = fabs(c_new - target), m0 = fabs(target - c);
                double mm = (m1 < m0 ? m1 : m0) / total;
                if (mm < g_margin[1]) g_margin[1] = mm;
                return j;
            }
            c = c_new;
            last = j;
        }
    }
    return last;
}

/* Accept / reject / resample for one sequence.
 * p_logits: k_eff+1 rows of n (target, after guidance); q_logits: k_eff rows (draft),
 * ignored when q_onehot (then q_i is the point mass on drafts[i]).
 * Draft i (0-based) is accepted iff u_acc[i] * q_i(d_i) < p_i(d_i), i.e. with probability
 * min(1, p/q); the scan stops at the first rejection.  a = number accepted.
 * a < k_eff : emit y ~ norm(max(0, p_a - q_a)) by inverse CDF with u_final (if that
 *             residual has no mass, y ~ p_a);
 * a == k_eff: emit the bonus token y ~ p_{k_eff}.
 * out_tokens[0..a-1] = accepted drafts, out_tokens[a] = y.  Returns a. */
int orc_spec_sample(int k_eff, int n, const float* p_logits, const float* q_logits,
                    const int32_t* drafts, int q_onehot, float temperature, int top_k,
                    const float* u_acc, float u_final, int32_t* out_tokens) {
    double* wp = (double*)malloc(sizeof(double) * (size_t)n);
    double* wq = (double*)malloc(sizeof(double) * (size_t)n);
    int a = 0, y = -1;
    for (; a < k_eff; ++a) {
        int dtok = drafts[a];
        double Zp = orc_warp(p_logits + (size_t)a * n, n, temperature, top_k, wp);
        double qd, Zq = 1.0;
        if (q_onehot) {
            qd = 1.0;
        } else {
            Zq = orc_warp(q_logits + (size_t)a * n, n, temperature, top_k, wq);
            qd = wq[dtok] / Zq;
        }
        double pd = wp[dtok] / Zp;
        double lhs = (double)u_acc[a] * qd;
        double mg = fabs(lhs - pd);
        if (mg < g_margin[0]) g_margin[0] = mg;
        if (lhs < pd) {
            out_tokens[a] = dtok;
            continue;
        }
        /* first rejection: residual distribution at this position */
        double R = 0.0;
        for (int j = 0; j < n; ++j) {
            double qj = q_onehot ? (j == dtok ? 1.0 : 0.0) : wq[j] / Zq;
            double r = wp[j] / Zp - qj;
            wq[j] = r > 0.0 ? r : 0.0;
            R += wq[j];
        }
        y = (R > 0.0) ? orc_inv_cdf(wq, n, R, u_final) : orc_inv_cdf(wp, n, Zp, u_final);
        break;
    }
    if (y < 0) {
        double Zp = orc_warp(p_logits + (size_t)k_eff * n, n, temperature, top_k, wp);
        y = orc_inv_cdf(wp, n, Zp, u_final);
    }
    out_tokens[a] = y;
    free(wp);
    free(wq);
    return a;
}

/* Several candidates at one position, each drawn from a proposal of its own (Method,
 * "Sampling and Verification", the recursion over consecutive rejections; appendix
 * "Theoretical Justification", general form with the ordered proposals q_1..q_m).
 * p^(1) = p.  Candidate i (1-based) is accepted with probability
 * min(1, p^(i)(s_i) / q_i(s_i)), decided as u_acc[i-1] * q_i(s_i) < p^(i)(s_i); after a
 * rejection p^(i+1) = norm(max(0, p^(i) - q_i)): the proposal subtracted is the rejected
 * candidate's own (the appendix's two-head case prints q_vert in both steps; its derivation
 * and the general form use q_i).  If a residual has no mass p^(i+1) = p^(i), as in
 * orc_spec_sample.  After m rejections the token is drawn from p^(m+1) by inverse CDF with
 * u_final.
 * p_logits: n; q_logits: m rows of n; cand: m tokens.  resid (may be NULL): m values, the
 * residual mass sum_x max(0, p^(i) - q_i) = 1 - alpha_i of every step that was evaluated
 * (steps after an acceptance: -1).
 * Returns the 0-based index of the accepted candidate, or m when all were rejected;
 * *out_token is the emitted token. */
int orc_multi_verify(int m, int n, const float* p_logits, const float* q_logits,
                     const int32_t* cand, float temperature, int top_k, const float* u_acc,
                     float u_final, int32_t* out_token, double* resid) {
    double* p = (double*)malloc(sizeof(double) * (size_t)n);
    double* q = (double*)malloc(sizeof(double) * (size_t)n);
    double Zp = orc_warp(p_logits, n, temperature, top_k, p);
    for (int j = 0; j < n; ++j) p[j] /= Zp;
    if (resid)
        for (int i = 0; i < m; ++i) resid[i] = -1.0;
    int acc = m;
    for (int i = 0; i < m; ++i) {
        double Zq = orc_warp(q_logits + (size_t)i * n, n, temperature, top_k, q);
        for (int j = 0; j < n; ++j) q[j] /= Zq;
        int s = cand[i];
        double lhs = (double)u_acc[i] * q[s];
        double mg = fabs(lhs - p[s]);
        if (mg < g_margin[0]) g_margin[0] = mg;
        double R = 0.0;
        for (int j = 0; j < n; ++j) {
            double r = p[j] - q[j];
            q[j] = r > 0.0 ? r : 0.0;   /* q now holds max(0, p^(i) - q_i) */
            R += q[j];
        }
        if (resid) resid[i] = R;
        if (lhs < p[s]) {
            acc = i;
            *out_token = s;
            break;
        }
        if (R > 0.0)
            for (int j = 0; j < n; ++j) p[j] = q[j] / R;
    }
    if (acc == m) {
        double total = 0.0;
        for (int j = 0; j < n; ++j) total += p[j];
        *out_token = orc_inv_cdf(p, n, total, u_final);
    }
    free(p);
    free(q);
    return acc;
}

/* ------------------------------------------------------------ model / state */

orc_model* orc_load(const void* blob, size_t nbytes, int samp_lo, int samp_n,
                    double rms_eps, double rope_theta) {
    if (!blob || nbytes < 64) return NULL;
    const int32_t* h = (const int32_t*)blob;
    if (h[0] != 0x4B574148 || h[1] != 1 || (h[2] != 0 && h[2] != 1)) return NULL;
    orc_model* M = (orc_model*)calloc(1, sizeof *M);
    M->dtype = h[2];
    M->L = h[3];
    M->d = h[4];
    M->H = h[5];
    M->m = h[6];
    M->V = h[7];
    if (M->L < 1 || M->d < 2 || M->H < 1 || M->d % M->H || (M->d / M->H) % 2 || M->m < 1 || M->V < 1) {
        free(M);
        return NULL;
    }
    M->hd = M->d / M->H;
    M->samp_lo = samp_lo;
    M->Vs = samp_n ? samp_n : M->V;
    if (samp_lo < 0 || M->Vs < 1 || samp_lo + M->Vs > M->V) {
        free(M);
        return NULL;
    }
    M->eps = rms_eps;
    M->theta = rope_theta;
    M->blob = (const uint8_t*)blob;
    M->esz = M->dtype == 0 ? 4 : 2;
    size_t d = (size_t)M->d, m = (size_t)M->m, V = (size_t)M->V, e = M->esz;
    size_t** per[9] = {&M->off_g1, &M->off_Wq, &M->off_Wk, &M->off_Wv, &M->off_Wo,
                       &M->off_g2, &M->off_W1, &M->off_W3, &M->off_W2};
    size_t cnt[9] = {d, d * d, d * d, d * d, d * d, d, m * d, m * d, d * m};
    for (int t = 0; t < 9; ++t) *per[t] = (size_t*)malloc(sizeof(size_t) * (size_t)M->L);
    size_t off = 64;
    M->off_E = off;
    off += V * d * e;
    for (int l = 0; l < M->L; ++l)
        for (int t = 0; t < 9; ++t) {
            (*per[t])[l] = off;
            off += cnt[t] * e;
        }
    M->off_gf = off;
    off += d * e;
    M->off_Wout = off;
    off += V * d * e;
    M->off_Wd = off;
    off += d * 3 * d * e;
    if (off != nbytes) {
        orc_free_model(M);
        return NULL;
    }
    return M;
}

void orc_free_model(orc_model* M) {
    if (!M) return;
    free(M->off_g1); free(M->off_Wq); free(M->off_Wk); free(M->off_Wv); free(M->off_Wo);
    free(M->off_g2); free(M->off_W1); free(M->off_W3); free(M->off_W2);
    free(M);
}

orc_state* orc_new_state(const orc_model* M, int batch, int use_cfg, int max_cond,
                         int grid_h, int grid_w, int k_max) {
    if (!M || batch < 1 || max_cond < 1 || grid_h < 1 || grid_w < 1 || k_max < 0 || k_max > 63)
        return NULL;
    orc_state* st = (orc_state*)calloc(1, sizeof *st);
    st->M = M;
    st->B = batch;
    st->use_cfg = use_cfg ? 1 : 0;
    st->S = batch * (use_cfg ? 2 : 1);
    st->Cmax = max_cond;
    st->gh = grid_h;
    st->gw = grid_w;
    st->N = grid_h * grid_w;
    st->kmax = k_max;
    st->Tmax = max_cond + st->N;
    size_t kv = (size_t)st->S * M->L * st->Tmax * M->d;
    st->Kc = (double*)malloc(sizeof(double) * kv);
    st->Vc = (double*)malloc(sizeof(double) * kv);
    st->grid = (int32_t*)calloc((size_t)st->B * st->N, 4);
    st->n = (int32_t*)calloc((size_t)st->B, 4);
    st->k_eff = (int32_t*)calloc((size_t)st->B, 4);
    st->draft = (int32_t*)calloc((size_t)st->B * (k_max + 1), 4);
    st->h_prev = (double*)calloc((size_t)st->S * M->d, 8);
    st->hid = (double*)calloc((size_t)st->S * (k_max + 1) * M->d, 8);
    st->lq = (float*)calloc((size_t)st->B * (k_max + 1) * M->Vs, 4);
    st->lp = (float*)calloc((size_t)st->B * (k_max + 1) * M->Vs, 4);
    if (!st->Kc || !st->Vc || !st->lq || !st->lp) {
        orc_free_state(st);
        return NULL;
    }
    return st;
}

void orc_free_state(orc_state* st) {
    if (!st) return;
    free(st->Kc); free(st->Vc); free(st->grid); free(st->n); free(st->k_eff);
    free(st->draft); free(st->h_prev); free(st->hid); free(st->lq); free(st->lp);
    free(st);
}

/* ------------------------------------------------------------ target forward */

/* One row through every layer.  Row at position pos attends cache entries 0..pos of its
 * own sequence (itself included), which is exactly causal attention; feeding the k+1
 * rows of a verify step one after another therefore realises the block-causal mask. */
int orc_forward_row(orc_state* st, int seq, int pos, double* x, float* logits) {
    const orc_model* M = st->M;
    if (seq < 0 || seq >= st->S || pos < 0 || pos >= st->Tmax) return ORC_EINVAL;
    int d = M->d, hd = M->hd, m = M->m;
    double* a = (double*)malloc(sizeof(double) * (size_t)d);
    double* q = (double*)malloc(sizeof(double) * (size_t)d);
    double* o = (double*)malloc(sizeof(double) * (size_t)d);
    double* t = (double*)malloc(sizeof(double) * (size_t)d);
    double* u1 = (double*)malloc(sizeof(double) * (size_t)m);
    double* u3 = (double*)malloc(sizeof(double) * (size_t)m);
    double* sc = (double*)malloc(sizeof(double) * (size_t)(pos + 1));
    for (int l = 0; l < M->L; ++l) {
        double* Kl = st->Kc + (((size_t)seq * M->L + l) * st->Tmax) * d;
        double* Vl = st->Vc + (((size_t)seq * M->L + l) * st->Tmax) * d;
        double* kpos = Kl + (size_t)pos * d;
        double* vpos = Vl + (size_t)pos * d;
        rmsnorm(M, M->off_g1[l], x, a);
        matvec(M, M->off_Wq[l], 0, d, d, a, q);
        matvec(M, M->off_Wk[l], 0, d, d, a, kpos);
        matvec(M, M->off_Wv[l], 0, d, d, a, vpos);
        rope(M, q, pos);
        rope(M, kpos, pos);
        double scale = 1.0 / sqrt((double)hd);
        for (int h = 0; h < M->H; ++h) {
            const double* qh = q + (size_t)h * hd;
            double mx = -INFINITY;
            for (int tt = 0; tt <= pos; ++tt) {
                const double* kh = Kl + (size_t)tt * d + (size_t)h * hd;
                double s = 0.0;
                for (int i = 0; i < hd; ++i) s += qh[i] * kh[i];
                sc[tt] = s * scale;
                if (sc[tt] > mx) mx = sc[tt];
            }
            double den = 0.0;
            for (int tt = 0; tt <= pos; ++tt) {
                sc[tt] = exp(sc[tt] - mx);
                den += sc[tt];
            }
            for (int i = 0; i < hd; ++i) {
                double acc = 0.0;
                for (int tt = 0; tt <= pos; ++tt) acc += sc[tt] * Vl[(size_t)tt * d + (size_t)h * hd + i];
                o[(size_t)h * hd + i] = acc / den;
            }
        }
        matvec(M, M->off_Wo[l], 0, d, d, o, t);
        for (int i = 0; i < d; ++i) x[i] += t[i];
        rmsnorm(M, M->off_g2[l], x, a);
        matvec(M, M->off_W1[l], 0, m, d, a, u1);
        matvec(M, M->off_W3[l], 0, m, d, a, u3);
        for (int i = 0; i < m; ++i) u1[i] = u1[i] / (1.0 + exp(-u1[i])) * u3[i]; /* silu(u1) * u3 */
        matvec(M, M->off_W2[l], 0, d, m, u1, t);
        for (int i = 0; i < d; ++i) x[i] += t[i];
    }
    if (logits) lm_head(M, x, logits);
    free(a); free(q); free(o); free(t); free(u1); free(u3); free(sc);
    return ORC_OK;
}

/* ------------------------------------------------------------ draft head */

/* g_out = W_d [g_prev | E[left] | E[up]] (up < 0: no upper neighbour, zeros); the draft
 * logits are the target's own final norm and output projection applied to g_out. */
int orc_draft_head(const orc_state* st, const double* g_prev, int left, int up, double* g_out,
                   float* logits) {
    const orc_model* M = st->M;
    int d = M->d;
    if (left < 0 || left >= M->V || up >= M->V) return ORC_EINVAL;
    double* in = (double*)malloc(sizeof(double) * 3 * (size_t)d);
    memcpy(in, g_prev, sizeof(double) * (size_t)d);
    embed(M, left, in + d);
    if (up >= 0) embed(M, up, in + 2 * d);
    else for (int i = 0; i < d; ++i) in[2 * d + i] = 0.0;
    matvec(M, M->off_Wd, 0, d, 3 * d, in, g_out);
    if (logits) lm_head(M, g_out, logits);
    free(in);
    return ORC_OK;
}

/* ------------------------------------------------------------ the step */

static int check_sampling_args(const orc_state* st, float temperature, int top_k, float cfg_scale) {
    if (!(temperature >= 0.0f) || top_k < 1 || top_k > st->M->Vs) return ORC_EINVAL;
    if (st->use_cfg ? (cfg_scale == 1.0f) : (cfg_scale != 1.0f)) return ORC_EINVAL;
    return ORC_OK;
}

int orc_prefill(orc_state* st, const float* cond, const float* uncond, int n_cond,
                float temperature, int top_k, float cfg_scale, const float* u_first) {
    if (!st || !cond || !u_first || n_cond < 1 || n_cond > st->Cmax) return ORC_EINVAL;
    if (check_sampling_args(st, temperature, top_k, cfg_scale)) return ORC_EINVAL;
    if (st->use_cfg && !uncond) return ORC_EINVAL;
    const orc_model* M = st->M;
    int d = M->d, Vs = M->Vs;
    st->C = n_cond;
    st->temperature = temperature;
    st->top_k = top_k;
    st->cfg_scale = cfg_scale;
    double* x = (double*)malloc(sizeof(double) * (size_t)d);
    float* lc = (float*)malloc(sizeof(float) * (size_t)Vs);
    float* lu = (float*)malloc(sizeof(float) * (size_t)Vs);
    double* w = (double*)malloc(sizeof(double) * (size_t)Vs);
    for (int b = 0; b < st->B; ++b) {
        for (int pass = 0; pass < (st->use_cfg ? 2 : 1); ++pass) {
            int s = pass ? st->B + b : b;
            const float* src = (pass ? uncond : cond) + (size_t)b * n_cond * d;
            for (int r = 0; r < n_cond; ++r) {
                for (int i = 0; i < d; ++i) x[i] = (double)src[(size_t)r * d + i];
                orc_forward_row(st, s, r, x, r == n_cond - 1 ? (pass ? lu : lc) : NULL);
            }
            memcpy(st->h_prev + (size_t)s * d, x, sizeof(double) * (size_t)d);
        }
        if (st->use_cfg) guide(lc, lu, cfg_scale, Vs, lc);
        double Z = orc_warp(lc, Vs, temperature, top_k, w);
        st->grid[(size_t)b * st->N] = M->samp_lo + orc_inv_cdf(w, Vs, Z, u_first[b]);
        st->n[b] = 1;
    }
    free(x); free(lc); free(lu); free(w);
    st->phase = 1;
    return ORC_OK;
}

/* Drafting phase.  With `forced` == NULL every draft is drawn from its own distribution
 * with u_draft; otherwise draft i is forced[b][i] (teacher-forced drafting: the head still
 * produces q_i from the forced left neighbours) and, if point_mass is set, q_i is replaced
 * by the point mass on that token (replay mode).  May be repeated before the verify call:
 * the last draft counts. */
static int draft_impl(orc_state* st, int k, const float* u_draft, const int32_t* forced, int point_mass,
                      int32_t* out_draft) {
    if (!st || k < 0 || k > st->kmax || k > st->gw) return ORC_EINVAL;
    if (k > 0 && !u_draft && !forced) return ORC_EINVAL;
    if (st->phase != 1 && st->phase != 2) return ORC_ESTATE;
    const orc_model* M = st->M;
    int d = M->d, Vs = M->Vs, N = st->N, IW = st->gw;
    if (forced)
        for (int b = 0; b < st->B; ++b) {
            int n = st->n[b];
            int ke = n >= N ? 0 : (k < N - n - 1 ? k : N - n - 1);
            for (int i = 0; i < ke; ++i) {
                int t = forced[(size_t)b * k + i];
                if (t < M->samp_lo || t >= M->samp_lo + Vs) return ORC_EINVAL;
            }
        }
    double* g = (double*)malloc(sizeof(double) * 2 * (size_t)d);
    double* gn = (double*)malloc(sizeof(double) * (size_t)d);
    float* lu = (float*)malloc(sizeof(float) * (size_t)Vs);
    double* w = (double*)malloc(sizeof(double) * (size_t)Vs);
    for (int b = 0; b < st->B; ++b) {
        int n = st->n[b];
        int32_t* dr = st->draft + (size_t)b * (st->kmax + 1);
        for (int i = 0; i < k; ++i) dr[i] = -1;
        if (out_draft)
            for (int i = 0; i < k; ++i) out_draft[(size_t)b * k + i] = -1;
        if (n >= N) {
            st->k_eff[b] = -1;
            continue;
        }
        int ke = k < N - n - 1 ? k : N - n - 1;
        st->k_eff[b] = ke;
        memcpy(g, st->h_prev + (size_t)b * d, sizeof(double) * (size_t)d);
        if (st->use_cfg) memcpy(g + d, st->h_prev + (size_t)(st->B + b) * d, sizeof(double) * (size_t)d);
        for (int i = 1; i <= ke; ++i) {
            int t = n - 1 + i; /* raster index this draft is for */
            int left = (i == 1) ? st->grid[(size_t)b * N + n - 1] : dr[i - 2];
            int up = (t >= IW) ? st->grid[(size_t)b * N + t - IW] : -1;
            float* lq = st->lq + ((size_t)b * (st->kmax + 1) + (i - 1)) * Vs;
            orc_draft_head(st, g, left, up, gn, lq);
            memcpy(g, gn, sizeof(double) * (size_t)d);
            if (st->use_cfg) {
                orc_draft_head(st, g + d, left, up, gn, lu);
                memcpy(g + d, gn, sizeof(double) * (size_t)d);
                guide(lq, lu, st->cfg_scale, Vs, lq);
            }
            if (forced) {
                dr[i - 1] = forced[(size_t)b * k + (i - 1)];
            } else {
                double Z = orc_warp(lq, Vs, st->temperature, st->top_k, w);
                dr[i - 1] = M->samp_lo + orc_inv_cdf(w, Vs, Z, u_draft[(size_t)b * k + (i - 1)]);
            }
        }
        if (out_draft)
            for (int i = 0; i < k; ++i) out_draft[(size_t)b * k + i] = dr[i];
    }
    free(g); free(gn); free(lu); free(w);
    st->k_last = k;
    st->q_onehot = (forced && point_mass) ? 1 : 0;
    st->phase = 2;
    return ORC_OK;
}

int orc_draft(orc_state* st, int k, const float* u_draft, int32_t* out_draft) {
    return draft_impl(st, k, u_draft, NULL, 0, out_draft);
}

int orc_draft_forced(orc_state* st, int k, const int32_t* tokens, int point_mass) {
    if (k > 0 && !tokens) return ORC_EINVAL;
    static const int32_t none = 0;
    return draft_impl(st, k, NULL, k > 0 ? tokens : &none, point_mass, NULL);
}

/* Feed rows [x_{n-1}, extra_0 .. extra_{cnt-2}] of prompt b through the target (both
 * streams), at positions C+n-1+r; keeps hidden rows and guided logits. */
static void target_rows(orc_state* st, int b, int rows, const int32_t* extra) {
    const orc_model* M = st->M;
    int d = M->d, Vs = M->Vs, n = st->n[b];
    double* x = (double*)malloc(sizeof(double) * (size_t)d);
    float* lu = (float*)malloc(sizeof(float) * (size_t)Vs);
    for (int r = 0; r < rows; ++r) {
        int tok = (r == 0) ? st->grid[(size_t)b * st->N + n - 1] : extra[r - 1];
        float* lp = st->lp + ((size_t)b * (st->kmax + 1) + r) * Vs;
        for (int pass = 0; pass < (st->use_cfg ? 2 : 1); ++pass) {
            int s = pass ? st->B + b : b;
            embed(M, tok, x);
            orc_forward_row(st, s, st->C + n - 1 + r, x, pass ? lu : lp);
            memcpy(st->hid + ((size_t)s * (st->kmax + 1) + r) * d, x, sizeof(double) * (size_t)d);
        }
        if (st->use_cfg) guide(lp, lu, st->cfg_scale, Vs, lp);
    }
    free(x);
    free(lu);
}

static void commit(orc_state* st, int b, const int32_t* toks, int cnt, int row) {
    const orc_model* M = st->M;
    int n = st->n[b], d = M->d;
    for (int i = 0; i < cnt; ++i) st->grid[(size_t)b * st->N + n + i] = toks[i];
    st->n[b] = n + cnt; /* cache entries beyond C + n - 1 are simply never read again */
    for (int pass = 0; pass < (st->use_cfg ? 2 : 1); ++pass) {
        int s = pass ? st->B + b : b;
        memcpy(st->h_prev + (size_t)s * d, st->hid + ((size_t)s * (st->kmax + 1) + row) * d,
               sizeof(double) * (size_t)d);
    }
}

int orc_verify(orc_state* st, int k, const float* u_acc, const float* u_final,
               int32_t* out_n_accept, int32_t* out_tokens) {
    if (!st || !u_final || (k > 0 && !u_acc)) return ORC_EINVAL;
    if (st->phase != 2 || k != st->k_last) return ORC_ESTATE;
    const orc_model* M = st->M;
    int Vs = M->Vs;
    int32_t toks[64];
    for (int b = 0; b < st->B; ++b) {
        int ke = st->k_eff[b];
        if (out_n_accept) out_n_accept[b] = -1;
        if (out_tokens)
            for (int i = 0; i <= k; ++i) out_tokens[(size_t)b * (k + 1) + i] = -1;
        if (ke < 0) continue;
        int32_t* dr = st->draft + (size_t)b * (st->kmax + 1);
        target_rows(st, b, ke + 1, dr);
        int32_t rel[64];
        for (int i = 0; i < ke; ++i) rel[i] = dr[i] - M->samp_lo;
        int a = orc_spec_sample(ke, Vs, st->lp + (size_t)b * (st->kmax + 1) * Vs,
                                st->lq + (size_t)b * (st->kmax + 1) * Vs, rel, st->q_onehot,
                                st->temperature, st->top_k, u_acc + (size_t)b * k, u_final[b], toks);
        for (int i = 0; i <= a; ++i) toks[i] += M->samp_lo;
        commit(st, b, toks, a + 1, a);
        if (out_n_accept) out_n_accept[b] = a;
        if (out_tokens)
            for (int i = 0; i <= a; ++i) out_tokens[(size_t)b * (k + 1) + i] = toks[i];
    }
    st->phase = 1;
    return ORC_OK;
}

/* Teacher forcing / re-synchronisation: rewind prompt b to n_from[b] committed tokens,
 * then commit tokens[b][0..cnt) as if all had been accepted. */
int orc_force(orc_state* st, const int32_t* n_from, const int32_t* tokens, int cnt) {
    if (!st || !n_from || !tokens || cnt < 1 || cnt > st->kmax + 1) return ORC_EINVAL;
    if (st->phase < 1) return ORC_ESTATE;
    for (int b = 0; b < st->B; ++b) {
        if (n_from[b] < 1 || n_from[b] > st->n[b] || n_from[b] + cnt > st->N) return ORC_EINVAL;
        for (int i = 0; i < cnt; ++i) {
            int t = tokens[(size_t)b * cnt + i];
            if (t < 0 || t >= st->M->V) return ORC_EINVAL;
        }
    }
    for (int b = 0; b < st->B; ++b) {
        st->n[b] = n_from[b];
        target_rows(st, b, cnt, tokens + (size_t)b * cnt);
        commit(st, b, tokens + (size_t)b * cnt, cnt, cnt - 1);
    }
    st->phase = 1;
    return ORC_OK;
}

int orc_generate(orc_state* st, const float* cond, const float* uncond, int n_cond, int k,
                 float temperature, int top_k, float cfg_scale, uint64_t seed,
                 int32_t* out_grid, int64_t* out_stats) {
    if (!st || k < 0 || k > st->kmax) return ORC_EINVAL;
    int B = st->B;
    float* u = (float*)calloc((size_t)B * (2 * (size_t)k + 2), sizeof(float));
    float *ud = u, *ua = u + (size_t)B * k, *uf = ua + (size_t)B * k;
    int32_t* na = (int32_t*)malloc(4 * (size_t)B);
    for (int b = 0; b < B; ++b) uf[b] = orc_uniform(seed, (uint32_t)b, 0, ORC_SLOT_FINAL);
    int rc = orc_prefill(st, cond, uncond, n_cond, temperature, top_k, cfg_scale, uf);
    int64_t steps = 0, accepted = 0, tokens = 0, iters = 0;
    for (uint32_t step = 1; rc == ORC_OK; ++step) {
        int active = 0;
        for (int b = 0; b < B; ++b) active += st->n[b] < st->N;
        if (!active) break;
        for (int b = 0; b < B; ++b) {
            for (int i = 0; i < k; ++i) {
                ud[(size_t)b * k + i] = orc_uniform(seed, (uint32_t)b, step, ORC_SLOT_DRAFT + (uint32_t)i);
                ua[(size_t)b * k + i] = orc_uniform(seed, (uint32_t)b, step, ORC_SLOT_ACC + (uint32_t)i);
            }
            uf[b] = orc_uniform(seed, (uint32_t)b, step, ORC_SLOT_FINAL);
        }
        rc = orc_draft(st, k, ud, NULL);
        if (rc == ORC_OK) rc = orc_verify(st, k, ua, uf, na, NULL);
        for (int b = 0; b < B && rc == ORC_OK; ++b)
            if (na[b] >= 0) {
                steps += 1;
                accepted += na[b];
                tokens += na[b] + 1;
            }
        iters += 1;
    }
    if (rc == ORC_OK && out_grid) memcpy(out_grid, st->grid, 4 * (size_t)B * st->N);
    if (out_stats) {
        out_stats[0] = steps;
        out_stats[1] = accepted;
        out_stats[2] = tokens;
        out_stats[3] = iters;
    }
    free(u);
    free(na);
    return rc;
}

/* ------------------------------------------------------------ inspection */

/* Threads the matrix-vector products run on. */
int orc_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}


int orc_get_n(const orc_state* st, int32_t* n) {
    if (!st || !n) return ORC_EINVAL;
    memcpy(n, st->n, 4 * (size_t)st->B);
    return ORC_OK;
}

int orc_get_grid(const orc_state* st, int32_t* grid) {
    if (!st || !grid) return ORC_EINVAL;
    memcpy(grid, st->grid, 4 * (size_t)st->B * st->N);
    return ORC_OK;
}

int orc_get_logits(const orc_state* st, float* out) {
    if (!st || !out) return ORC_EINVAL;
    int rows = st->k_last + 1, Vs = st->M->Vs;
    for (int b = 0; b < st->B; ++b)
        memcpy(out + (size_t)b * rows * Vs, st->lp + (size_t)b * (st->kmax + 1) * Vs,
               sizeof(float) * (size_t)rows * Vs);
    return ORC_OK;
}

int orc_get_draft_logits(const orc_state* st, float* out) {
    if (!st || !out) return ORC_EINVAL;
    int rows = st->k_last, Vs = st->M->Vs;
    for (int b = 0; b < st->B; ++b)
        memcpy(out + (size_t)b * rows * Vs, st->lq + (size_t)b * (st->kmax + 1) * Vs,
               sizeof(float) * (size_t)rows * Vs);
    return ORC_OK;
}

int orc_get_hprev(const orc_state* st, double* out) {
    if (!st || !out) return ORC_EINVAL;
    memcpy(out, st->h_prev, sizeof(double) * (size_t)st->S * st->M->d);
    return ORC_OK;
}
