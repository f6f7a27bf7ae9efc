/*
 * CPU oracle for one speculate-and-verify step of spatially-conditioned speculative
 * decoding of autoregressive image tokens (Hawk, arXiv 2510.25739).
 *
 * TEST INFRASTRUCTURE ONLY.  Plain, slow, obviously-correct C, fp64 arithmetic on the
 * weight values as stored.  It shares no code with the HIP library and must never be
 * called from the product path: only tests, the smoke check and the benchmark's CPU
 * baseline leg may use it.
 *
 * What the paper fixes and this file follows:
 *   - raster-order next-token factorisation (Preliminary, "Autoregressive Image
 *     Generation");
 *   - draft, one target pass over all drafted positions, accept each draft with
 *     probability min(1, p/q), resample the first rejected position from
 *     norm(max(0, p - q)) (Preliminary, "Speculative Sampling"; Method, "Sampling and
 *     Verification", the recursion for consecutive rejections with one candidate per
 *     depth);
 *   - draft heads sit on the target's final hidden state and reuse its output
 *     projection (Preliminary, "Utilization of Draft Heads Structure"; appendix "Draft
 *     Heads Structure and Memory Overhead"), and read the spatial neighbours
 *     x_{T-1} and x_{T-IW} (Preliminary, "Attention Sinking");
 *   - top-k / temperature sampling and classifier-free guidance (Experiment, "Model and
 *     Benchmark").
 * The target decoder's internals (pre-RMSNorm, RoPE, SwiGLU) are not described by the
 * paper; they follow the workload definitions this build was given.
 *
 * Pinned by tests/test_oracle_*.py: greedy speculative == plain AR; chi-square of the
 * emitted token against p; exact enumeration of accept/reject paths with rational
 * arithmetic; acceptance rate == sum min(p,q); residual identity; softmax / argmax
 * special cases of the warp; the multi-candidate recursion by exact integration over its
 * uniforms (output law == p for distinct proposals) and its one-candidate case against
 * orc_spec_sample; incremental KV forward == full causal recompute and ==
 * an independent PyTorch fp64 forward; hand-computed draft head.
 * Parity unpinned: behaviour with trained weights (accept length, FID, CLIP).
 */
#ifndef HAWK_ORACLE_H
#define HAWK_ORACLE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct orc_model orc_model;
typedef struct orc_state orc_state;

enum { ORC_OK = 0, ORC_EINVAL = -1, ORC_ESTATE = -2, ORC_ENOMEM = -3 };

/* Slots of the counter-based uniform generator used by orc_generate. */
enum { ORC_SLOT_DRAFT = 0, ORC_SLOT_ACC = 64, ORC_SLOT_FINAL = 128 };

/* The blob is borrowed (not copied): it must outlive the model. samp_n == 0 selects
 * the whole vocabulary. */
orc_model* orc_load(const void* blob, size_t nbytes, int samp_lo, int samp_n,
                    double rms_eps, double rope_theta);
void orc_free_model(orc_model*);

orc_state* orc_new_state(const orc_model*, int batch, int use_cfg, int max_cond,
                         int grid_h, int grid_w, int k_max);
void orc_free_state(orc_state*);

int orc_prefill(orc_state*, const float* cond, const float* uncond, int n_cond,
                float temperature, int top_k, float cfg_scale, const float* u_first);
int orc_draft(orc_state*, int k, const float* u_draft, int32_t* out_draft);
int orc_draft_forced(orc_state*, int k, const int32_t* tokens, int point_mass);
int orc_verify(orc_state*, int k, const float* u_acc, const float* u_final,
               int32_t* out_n_accept, int32_t* out_tokens);
int orc_force(orc_state*, const int32_t* n_from, const int32_t* tokens, int cnt);
int orc_generate(orc_state*, const float* cond, const float* uncond, int n_cond, int k,
                 float temperature, int top_k, float cfg_scale, uint64_t seed,
                 int32_t* out_grid, int64_t* out_stats /* steps, accepted, tokens, iters */);

/* State inspection. */
int orc_num_threads(void);
int orc_get_n(const orc_state*, int32_t* n /*[batch]*/);
int orc_get_grid(const orc_state*, int32_t* grid /*[batch, N]*/);
int orc_get_logits(const orc_state*, float* out /*[batch, k_last+1, V_s]*/);
int orc_get_draft_logits(const orc_state*, float* out /*[batch, k_last, V_s]*/);
int orc_get_hprev(const orc_state*, double* out /*[n_seq, d]*/);

/* Building blocks, exported so that the tests can pin each one separately. */
float orc_uniform(uint64_t seed, uint32_t seq, uint32_t step, uint32_t slot);
double orc_warp(const float* logits, int n, float temperature, int top_k, double* w);
int orc_inv_cdf(const double* w, int n, double total, float u);
int orc_spec_sample(int k_eff, int n, const float* p_logits, const float* q_logits,
                    const int32_t* drafts, int q_onehot, float temperature, int top_k,
                    const float* u_acc, float u_final, int32_t* out_tokens);
/* m candidates at one position, each from its own proposal: sequential accept tests with
 * the recursively updated target p^(i+1) = norm(max(0, p^(i) - q_i)); see the definition. */
int orc_multi_verify(int m, int n, const float* p_logits, const float* q_logits,
                     const int32_t* cand, float temperature, int top_k, const float* u_acc,
                     float u_final, int32_t* out_token, double* resid);
/* One target row: x (d values: in = input embedding, out = hidden before the final
 * norm) at absolute position pos of sequence seq; appends K,V; logits may be NULL. */
int orc_forward_row(orc_state*, int seq, int pos, double* x, float* logits);
/* Classifier-free guidance on logit rows, as every guided row of the oracle is formed:
 * out = lu + scale * (lc - lu). */
void orc_guide(const float* lc, const float* lu, float scale, int n, float* out);
int orc_draft_head(const orc_state*, const double* g_prev, int left, int up, double* g_out,
                   float* logits);

/* Smallest decision margins seen since the last reset: [0] |u*q - p| of an accept test,
 * [1] |u*Z - cumsum| / Z of an inverse-CDF draw, [2] gap between the last kept and the
 * first dropped scaled logit of a top-k cut. */
void orc_margins(double out[3], int reset);

#ifdef __cplusplus
}
#endif
#endif
