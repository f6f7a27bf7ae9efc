/*
 * hawk.h - C ABI of the MI355X (gfx950) library for the hot path of Hawk-style
 * speculative decoding of autoregressive image tokens (arXiv 2510.25739).
 *
 * One step of the path = draft k tokens with a spatially conditioned head, score all
 * k+1 positions in one pass of the target decoder over its KV cache, then run the fused
 * speculative-sampling stage (top-k softmax, accept with min(1, p/q), resample the
 * first rejected position from norm(max(0, p - q))).
 *
 * Conventions for every entry point
 *   - Returns HAWK_OK (0) or a negative error code; never throws, never aborts.
 *     hawk_last_error() returns a text for the last failure on that context.
 *   - "host" pointers are ordinary CPU memory owned by the caller and are only read or
 *     written during the call.  "device" pointers are GPU memory owned by the caller.
 *   - The library allocates no device memory: all of it lives in the workspace the
 *     caller hands to hawk_create (size from hawk_workspace_bytes) and must stay valid
 *     and untouched until hawk_destroy.
 *   - Work is enqueued on the HIP stream given to hawk_create.  A call that has host
 *     outputs synchronises that stream before it returns; with all outputs NULL it
 *     returns as soon as the work is enqueued.
 *   - A context is not thread safe.  Call order: create, load, then per image
 *     prefill, (draft | draft_forced, verify)*  - or generate, which does all of that.
 *   - Token ids are full-vocabulary ids.  Sampling is restricted to the contiguous id
 *     range [samp_lo, samp_lo + samp_n); logit rows have samp_n entries.
 *   - Sequences: `batch` prompts; with classifier-free guidance (cfg_scale != 1) every
 *     prompt has a conditional and an unconditional stream (2*batch sequences).
 *   - Uniforms are fp32 in [0, 1).
 */
#ifndef HAWK_H
#define HAWK_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct hawk_ctx hawk_ctx;

enum {
    HAWK_OK = 0,
    HAWK_EINVAL = -1,  /* bad argument */
    HAWK_ESTATE = -2,  /* call out of order */
    HAWK_ENOMEM = -3,  /* workspace too small */
    HAWK_EDEVICE = -4  /* HIP runtime error, or a wait inside a persistent kernel ran out (the context is dead then) */
};

enum { HAWK_FP32 = 0, HAWK_BF16 = 1 };

/* Shape of the target decoder (pre-RMSNorm, rotary positions, SwiGLU MLP, no biases),
 * of the sampled vocabulary slice, and the capacity limits of one context.
 * dtype is the storage type of the weight blob: HAWK_FP32 computes with fp64
 * accumulators and activations (the exact-parity configuration), HAWK_BF16 with bf16
 * weights, a 16-bit (fp16) KV cache, fp32 accumulators and residual stream. */
typedef struct {
    int32_t n_layers, d_model, n_heads, d_mlp, vocab;
    int32_t samp_lo, samp_n;              /* samp_n == 0: whole vocabulary */
    int32_t max_cond, max_grid_h, max_grid_w, max_batch, k_max;
    int32_t dtype;                        /* HAWK_FP32 or HAWK_BF16 */
    int32_t use_cfg;                      /* 1: contexts run two streams per prompt */
    float rms_eps, rope_theta;
} hawk_config;

/* Counters of one hawk_generate call.  steps = prompt-steps executed (one per prompt
 * per speculate-and-verify step while the prompt was unfinished), accepted = drafts
 * accepted, tokens = image tokens committed by those steps (accepted + steps), iters =
 * lock-step iterations of the batch.  Accept length (Experiment, "Metrics") is
 * tokens / steps.  Times are milliseconds of GPU time on the context's stream. */
typedef struct {
    int64_t steps, accepted, tokens, iters;
    float ms_prefill, ms_decode;
} hawk_stats;

/* Bytes of device workspace a context of this configuration needs; 0 if the
 * configuration is invalid. */
size_t hawk_workspace_bytes(const hawk_config* cfg);

/* Host-only diagnostic of how the persistent weight-streaming kernel would split this
 * configuration over its workgroups (no GPU needed).  out8 (host, 8 x int64): [0] 1 if the
 * shape is supported by that kernel, [1] 1 KB weight tiles per layer, [2] tiles in total,
 * [3] / [4] fewest / most tiles one workgroup streams per layer, [5] rounds of the output
 * projection, [6] 1 if the job tables cover every tile exactly once, [7] workgroups. */
int hawk_plan_info(const hawk_config* cfg, int64_t* out8);

/* Creates a context over `workspace` (device, 256-byte aligned, >= hawk_workspace_bytes)
 * that enqueues on `hip_stream` (a hipStream_t, NULL = the default stream). */
int hawk_create(const hawk_config* cfg, void* workspace, size_t workspace_bytes,
                void* hip_stream, hawk_ctx** out);
void hawk_destroy(hawk_ctx* ctx);
const char* hawk_last_error(const hawk_ctx* ctx);

/* hawk_load(weights): copies a weight blob (host) into the workspace and prepares the
 * device layouts.  Blob = 64-byte header of int32 {magic 'HAWK', version 1, dtype,
 * n_layers, d_model, n_heads, d_mlp, vocab, 0...} followed by row-major [out, in]
 * tensors in dtype: E[vocab,d]; per layer g1[d] Wq Wk Wv Wo [d,d] g2[d] W1 W3 [m,d]
 * W2[d,m]; g_f[d]; W_out[vocab,d]; W_d[d,3d].  The draft head is one linear map over
 * [previous head output or target hidden | embedding of the left neighbour | embedding
 * of the upper neighbour] followed by the target's own final norm and output projection
 * (draft heads on the final hidden state: Preliminary, "Utilization of Draft Heads
 * Structure"; spatial neighbours x_{T-1}, x_{T-IW}: Preliminary, "Attention Sinking").
 * Header fields must match the context's configuration.  For bf16 the workspace then holds
 * the blob plus re-tiled copies of the GEMM weights in MFMA operand order (one for the
 * persistent kernel where it covers the shape, one tile-major copy for the other GEMM kernels):
 * hawk_workspace_bytes accounts for them. */
int hawk_load(hawk_ctx* ctx, const void* host_blob, size_t nbytes);

/* hawk_prefill(cond): runs the target over the condition vectors (host, fp32
 * [batch, n_cond, d]; uncond likewise or NULL without guidance), fills the KV cache,
 * samples image token 0 of every prompt with u_first (host [batch]) and fixes the
 * decoding parameters of this image: grid size, temperature (0 = greedy), top_k in
 * [1, samp_n], cfg_scale (== 1 exactly iff the context was created without use_cfg;
 * guided logits are l_u + s (l_c - l_u)).  Top-k / temperature / guidance: Experiment,
 * "Model and Benchmark".  Raster order: Preliminary, "Autoregressive Image
 * Generation". */
int hawk_prefill(hawk_ctx* ctx, const float* cond, const float* uncond, int batch, int n_cond,
                 int grid_h, int grid_w, float temperature, int top_k, float cfg_scale,
                 const float* u_first);

/* hawk_draft(k): the drafting phase (Preliminary, "Speculative Sampling").  For each
 * unfinished prompt drafts k_eff = min(k, N - n - 1) tokens for raster positions
 * n .. n+k_eff-1 (n = tokens committed so far), one after another: draft i reads the
 * previous head output (the target's hidden state for i = 1), the embedding of the token
 * left of its position (the previous draft for i > 1) and of the token above it (zeros
 * on the first image row), and is sampled by inverse CDF with u_draft (host [batch, k])
 * from the top-k/temperature-warped, guided draft logits.  k <= k_max and k <= grid_w.
 * out_draft (host [batch, k], may be NULL) receives the tokens, -1 where none. */
int hawk_draft(hawk_ctx* ctx, int k, const float* u_draft, int32_t* out_draft);

/* Teacher-forced drafting: like hawk_draft, but draft i of prompt b is tokens[b][i]
 * (host [batch, k], ids inside the sampled slice) instead of a draw; the head still runs
 * and produces q_i from the forced left neighbours.  point_mass != 0 replaces q_i by the
 * point mass on the forced token (replay mode: acceptance probability p_i(d_i)).
 * hawk_draft / hawk_draft_forced may be repeated before hawk_verify; the last one counts. */
int hawk_draft_forced(hawk_ctx* ctx, int k, const int32_t* tokens, int point_mass);

/* hawk_verify(k): the verification phase (Preliminary, "Speculative Sampling"; Method,
 * "Sampling and Verification" with one candidate per depth).  One target pass over the
 * rows [last committed token, draft 1 .. draft k_eff] of every sequence, appended to
 * the KV cache under a block-causal mask; then, per prompt, draft i is accepted iff
 * u_acc[i] * q_i(d_i) < p_i(d_i) (probability min(1, p/q)), stopping at the first
 * rejection; a = number accepted.  If a < k_eff the next token is drawn with u_final
 * from norm(max(0, p_{a+1} - q_{a+1})), else from p_{k_eff+1}.  Commits a+1 tokens,
 * drops the rejected rows from the cache and keeps the hidden state of row a for the
 * next draft.  u_acc host [batch, k], u_final host [batch]; out_n_accept host [batch]
 * (-1 for a finished prompt) and out_tokens host [batch, k+1] (-1 padded) may be NULL. */
int hawk_verify(hawk_ctx* ctx, int k, const float* u_acc, const float* u_final,
                int32_t* out_n_accept, int32_t* out_tokens);

/* hawk_generate(cond, grid_h, grid_w, k, temperature, top_k, cfg_scale, seed): prefill,
 * then draft + verify until every prompt has grid_h * grid_w tokens.  Uniforms come from
 * a counter-based generator: u(seed, prompt b, step s, slot) = top 24 bits of
 * mix(mix(seed + G) + G * (((b << 44) | (s << 8) | slot) + 1)) / 2^24 with mix the
 * splitmix64 finaliser and G = 0x9E3779B97F4A7C15; slot = i for draft i, 64 + i for
 * acceptance test i, 128 for the resample/bonus draw; step 0 slot 128 samples token 0,
 * steps count from 1.  replay_tokens (host [batch, N] or NULL) switches to replay mode:
 * the head still runs, but draft i of a step is replay_tokens[b][n + i - 1] with a
 * point-mass draft distribution.
 * out_grid host [batch, N]; stats may be NULL. */
int hawk_generate(hawk_ctx* ctx, const float* cond, const float* uncond, int batch, int n_cond,
                  int grid_h, int grid_w, int k, float temperature, int top_k, float cfg_scale,
                  uint64_t seed, const int32_t* replay_tokens, int32_t* out_grid,
                  hawk_stats* stats);

/* Runs n_steps speculate-and-verify steps (draft + verify) from the current state with
 * generator uniforms (seed; the step counter continues from the context's), without host
 * outputs: the benchmark's timed region.  replay != 0 drafts from the table given to the
 * last hawk_generate / hawk_set_replay in point-mass mode.  Steps after every prompt has
 * finished do nothing.  If ms_draft / ms_verify (host, single floats) are both non-NULL the
 * two phases are bracketed by events, the call synchronises and returns the summed GPU
 * milliseconds of each phase - and in ms_kernel (may be NULL) those of the persistent
 * target-pass kernel alone (0 if the generic kernels ran); otherwise it returns once the
 * work is enqueued. */
int hawk_run_steps(hawk_ctx* ctx, int k, int n_steps, uint64_t seed, int replay, float* ms_draft,
                   float* ms_verify, float* ms_kernel);

/* Stores the replay table (host [batch, N]) used by hawk_run_steps(replay = 1). */
int hawk_set_replay(hawk_ctx* ctx, const int32_t* replay_tokens);

/* Counters accumulated since the last hawk_prefill (times are left zero). */
int hawk_get_stats(hawk_ctx* ctx, hawk_stats* out);

/* Teacher forcing / re-synchronisation: rewinds prompt b to n_from[b] committed tokens
 * (1 <= n_from[b] <= current n) and commits tokens[b][0..cnt) as if all had been
 * accepted (cnt <= k_max + 1): runs the target over them, extends the cache, keeps the
 * hidden state of the last row.  n_from host [batch], tokens host [batch, cnt]. */
int hawk_force(hawk_ctx* ctx, const int32_t* n_from, const int32_t* tokens, int cnt);

/* State read-back (all host outputs, each synchronises the stream). */
int hawk_get_n(hawk_ctx* ctx, int32_t* n /*[batch]*/);
int hawk_get_grid(hawk_ctx* ctx, int32_t* grid /*[batch, N]*/);
/* guided target logits of the last verify/force, [batch, rows, samp_n], rows = k+1 or cnt */
int hawk_get_logits(hawk_ctx* ctx, float* out, int rows);
/* guided draft logits of the last draft, [batch, k, samp_n] */
int hawk_get_draft_logits(hawk_ctx* ctx, float* out, int k);

/* Selects the kernel set: 0 = one kernel per operation (any shape); 1 = a persistent
 * weight-streaming kernel where the shape allows (default): the one laid out on the chip's XCDs
 * for passes of at most 16 rows (step rows of hawk_verify / hawk_force / hawk_generate /
 * hawk_run_steps, tree rows of hawk_verify_tree; shapes: d_model 768, 1280 or - with the weights
 * streamed, at most 14 rows - 4096 with heads of 128), else the one with grid barriers; 2 = as 1 but
 * only the grid-barrier kernel.  hawk_last_path reports what the
 * last target pass actually used (0: one kernel per operation, 1: a persistent kernel; -1 before
 * any), hawk_last_kernel which kernel (0: one per operation, 1: grid-barrier kernel, 2: the kernel
 * laid out on the XCDs). */
int hawk_set_path(hawk_ctx* ctx, int path);
int hawk_last_path(const hawk_ctx* ctx);
int hawk_last_kernel(const hawk_ctx* ctx);

/* Error behaviour of the persistent kernels: every wait inside them (grid barriers, polls for partial
 * sums and flags) is bounded; a wait that runs out sets an error word in the workspace, the kernel
 * runs to its end without waiting any further, and the next call that returns data to the host
 * (hawk_draft with out_draft, hawk_verify with outputs, hawk_verify_tree, hawk_force, hawk_generate,
 * hawk_run_steps, every hawk_get_*) returns HAWK_EDEVICE.  From then on the context is dead: the
 * kernels' exchange buffers hold a mixture of two steps, so every further call on it returns
 * HAWK_EDEVICE at once without launching anything; destroy it and create a new one (the workspace
 * may be reused).
 *
 * Test hook: sets that error word from the host, as a timed-out wait would (no kernel is launched;
 * HAWK_ESTATE if the context's shape has no persistent-kernel plan). */
int hawk_debug_raise_timeout(hawk_ctx* ctx);

/* Diagnostic: switches per-stage time stamps of the streaming kernel on or off (they cost
 * a few stores per stage) and, if out != NULL, copies the stamps of the last launch to
 * out (host, n_words x uint64, at most 4*4096*8 + 2*256*256): [trace][stage][8] with trace 0, 1 = first
 * IO wave of workgroups 0 and 128 - 100 MHz ticks at: stage entry, barrier crossed, input
 * staged, workgroup sync 1, workgroup sync 2 (MFMAs done), results stored, arrival posted -
 * and trace 2, 3 = first compute wave of the same workgroups: stage entry, weight loads
 * issued, workgroup sync 1, weights landed, MFMAs done, partial sums handed over.  Behind
 * these 4*4096*8 words follow [2][256][256] words: for each of the first 256 stages, every
 * workgroup's arrival time at the stage's barrier, then the time it saw the previous
 * barrier's release. */
int hawk_phase_trace(hawk_ctx* ctx, int enable, uint64_t* out, size_t n_words);

/* Tree verification (Method, "Spatial Sampling Pool": the candidate tree is the Cartesian product
 * of the candidates of the positions ahead; "Sampling and Verification": candidates of one depth
 * are verified in order, an acceptance moves one depth down, a rejection of all of them ends the
 * step with a draw from the updated target).  Takes the place of hawk_draft + hawk_verify for one
 * step (call it after hawk_prefill, hawk_verify, hawk_force or itself).
 *   depth D (1..8) positions ahead; m_depth [D] (host) candidates per depth; the tree has
 *   1 + m_1 + m_1 m_2 + ... nodes (the root is the last committed token), at most 64 and at most
 *   k_max + 1 (the rows a context has room for); every unfinished prompt needs that many free
 *   positions left in its image (HAWK_EINVAL otherwise: finish with hawk_draft / hawk_verify).
 *   cand (host) [D][batch][m_max], m_max = max m_depth: candidate s of depth j + 1 as an index into
 *   the sampled slice; q_logits (DEVICE) [D][batch][m_max][V_s] fp32: the proposal each candidate
 *   was drawn from (e.g. the members of hawk_spec_pool); u_acc (host) [D][batch][m_max], u_final
 *   (host) [D + 1][batch] in [0, 1): u_final[j] draws the token after a rejection at depth j + 1,
 *   u_final[D] the extra token after D acceptances.  Entries beyond m_depth[j] are not read.
 * One target pass scores every node: node r's row sits at the root's position plus its depth and
 * attends the committed entries, its ancestors and itself (its keys and values go to the cache
 * entry root + r); the walk applies hawk_multi_verify's rule at each depth to the row of the node
 * it stands on; then the accepted path's cache entries are moved to their positions, tokens, n and
 * the hidden state for the next draft are committed as by hawk_verify.
 * out_n_accept (host, may be NULL) [batch]: candidates accepted (-1: prompt finished before the
 * call); out_tokens (host, may be NULL) [batch][D + 1]: the accepted + 1 tokens emitted (vocabulary
 * ids), -1 beyond.  Passes of at most 16 rows in all (sequences x nodes) of the shapes the
 * persistent kernel takes run on it, compiled with tree rows; larger ones run one kernel per
 * operation (hawk_last_path tells which).  With classifier-free guidance both streams of a prompt
 * go through the pass with the same tree and every target row is the guided combination, as in
 * hawk_verify.  The walk runs on the device; the call synchronises the stream twice (reading the
 * prompts' positions before, the results after).  depth x m_max <= 512.
 * hawk_get_tree_logits: the (guided) rows of the last tree pass, out (host)
 * [batch][n_nodes][V_s]. */
/* The order hawk_verify_tree gives the tree's nodes (host arithmetic only, all pointers host, each
 * out array may be NULL, room for 64 entries): node 0 is the root; then depth by depth every
 * combination of the candidates so far, the children of a node next to each other in candidate
 * order.  out_parent (-1 for the root), out_depth, out_candidate (which candidate of its depth; -1
 * for the root), out_ancestors (bit j set: node j lies on the path from the root, root included).
 * Returns the number of nodes, -1 for a bad shape (depth outside 1..8, a depth without candidates,
 * more than 64 nodes). */
int hawk_tree_layout(int depth, const int32_t* m_depth, int32_t* out_parent, int32_t* out_depth, int32_t* out_candidate,
                     uint64_t* out_ancestors);
int hawk_verify_tree(hawk_ctx* ctx, int depth, const int32_t* m_depth, const int32_t* cand, const float* q_logits,
                     const float* u_acc, const float* u_final, int32_t* out_n_accept, int32_t* out_tokens);
int hawk_get_tree_logits(hawk_ctx* ctx, float* out, int n_nodes);
/* The accepted path of the last tree step: out (host) [batch][8], entry j = node index of the
 * candidate accepted at depth j + 1 (valid for j < accepted count). */
int hawk_get_tree_path(hawk_ctx* ctx, int32_t* out);
/* Where the last target pass (hawk_verify, hawk_verify_tree, hawk_force) left the hidden states of
 * its rows - the final layer's output before the final norm, which draft heads read (Preliminary,
 * "Utilization of Draft Heads Structure"): *device_ptr points into the context's workspace, rows
 * [sequence][row of the pass][d_model], contiguous, elements of *elem_bytes bytes (4: fp32 in the
 * bf16 configurations, 8: fp64 in the fp32 configuration).  Valid until the next call that runs a
 * pass; the caller must not write there. */
int hawk_last_hidden(hawk_ctx* ctx, const void** device_ptr, int* elem_bytes);

/* Verification of several candidates at one position, each drawn from a proposal of its own
 * (Method, "Sampling and Verification": the iterated update of the target after consecutive
 * rejections; appendix "Theoretical Justification": general form for an ordered sequence of
 * proposals q_1..q_m, e.g. the vertical head's candidate first, then the horizontal one's).
 * For each of `rows` independent positions r:
 *   p^(1) = warp(p_logits[r]); for i = 1..m: q_i = warp(q_logits[r][i-1]), s_i = cand[r][i-1];
 *   s_i is accepted iff u_acc[r][i-1] * q_i(s_i) < p^(i)(s_i), i.e. with probability
 *   min(1, p^(i)(s_i) / q_i(s_i)); on rejection p^(i+1) = norm(max(0, p^(i) - q_i)) (p^(i) itself
 *   if that residual has no mass).  After m rejections the token is drawn from p^(m+1) by
 *   inverse CDF over ascending token index with u_final[r].
 * warp = temperature and top-k as in hawk_prefill (temperature 0 or top_k 1: point mass on the
 * arg-max); probabilities and sums in fp64.
 * All pointers are DEVICE pointers, rows contiguous: p_logits [rows][n] fp32, q_logits
 * [rows][m][n] fp32, cand [rows][m] (0 <= token < n; a value outside that range is rejected like a
 * token without target mass and nothing is read through it), u_acc [rows][m] and u_final [rows] in
 * [0, 1), out_index [rows] (0-based index of the accepted candidate, m if none), out_token
 * [rows], out_resid (may be NULL) [rows][m] fp64: the residual mass sum_x max(0, p^(i) - q_i)
 * = 1 - acceptance probability of every evaluated step, -1 for steps after an acceptance.
 * m_rows (device, may be NULL) [rows]: the number of candidates position r really has, clamped to
 * 0..m (a sampling pool near the top of the image has fewer members); candidates, proposals and
 * uniforms beyond it are not read, out_index[r] is then that count if none was accepted, and with
 * no candidate at all the token is drawn from the warped target itself.
 * n <= 16384.  workspace (device, may be NULL): with at least
 * hawk_multi_verify_workspace_bytes(rows, m) bytes the top-k selections of the target row and of
 * the m proposal rows of every position run in parallel workgroups (two launches) instead of one
 * after the other; the results are identical.  The caller owns every buffer; nothing is
 * allocated.  The launches are asynchronous on `stream` (a hipStream_t, NULL: the default
 * stream).
 * Returns HAWK_OK, HAWK_EINVAL (null pointer, m < 1, n out of range, top_k < 1, negative
 * temperature) or HAWK_EDEVICE (a launch failed). */
size_t hawk_multi_verify_workspace_bytes(int rows, int m);
int hawk_multi_verify(const float* p_logits, const float* q_logits, const int32_t* cand, const float* u_acc,
                      const float* u_final, const int32_t* m_rows, int rows, int m, int n, float temperature, int top_k,
                      int32_t* out_index, int32_t* out_token, double* out_resid, void* workspace,
                      size_t workspace_bytes, void* stream);

/* hawk_multi_verify for callers that cannot allocate device memory (code under HIP graph capture, tight
 * serving loops, harnesses that forbid allocation): the same operation, arguments, kernels and
 * results as hawk_multi_verify with a workspace, but the rows' statistics are kept in a fixed array
 * of 96 KiB that the library holds in device memory (one copy per GPU for the life of the process)
 * instead of a caller-provided buffer.  Nothing is allocated or freed by the call.
 * Limit: rows * (m + 1) <= 4096 logit rows per call; beyond it HAWK_ENOMEM is returned and nothing is
 * launched.  All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (two
 * streams, two threads) race and must be serialised by the caller; calls on one stream are ordered.
 * Nothing in the array has to be cleared between calls.  Other return codes as hawk_multi_verify. */
int hawk_multi_verify_static(const float* p_logits, const float* q_logits, const int32_t* cand, const float* u_acc,
                             const float* u_final, const int32_t* m_rows, int rows, int m, int n, float temperature,
                             int top_k, int32_t* out_index, int32_t* out_token, double* out_resid, void* stream);

/* ---- Spatial drafting structures ------------------------------------------------------------
 * Method, "Dual Direction Drafting Heads" and "Spatial Sampling Pool"; appendix "Draft Heads
 * Structure and Memory Overhead".  Positions count in raster order (position = row * IW +
 * column); T below is the position a hidden state predicts through the model's own output layer.
 * These entry points need no context: all pointers are DEVICE pointers unless stated, the caller
 * owns every buffer, nothing is allocated, launches are asynchronous on `stream` (a hipStream_t,
 * NULL: the default stream). */

/* Dual-direction draft heads.  Head j is a linear layer of the hidden size with SiLU, added back
 * to its input (the Medusa block the appendix names), and all heads share the model's output
 * layer:  g[r][j] = h[r] + silu(W_heads[j] h[r]),  q_logits[r][j] = W_out g[r][j].
 * The caller decides which heads are horizontal (head for T + j) and which vertical (T + d * IW).
 * h [rows][d] fp32; W_heads [n_heads][d][d] bf16, [out][in]; W_out [V_s][d] bf16 (the rows of the
 * output layer that are sampled from); q_logits [rows][n_heads][V_s] fp32; g_out (may be NULL)
 * [rows][n_heads][d] fp32.  Products on the matrix units: activations as two bf16 planes (about 16
 * bits), fp32 accumulation.  d % 64 == 0, V_s % 16 == 0, pointers 16-byte aligned; workspace of at
 * least hawk_spatial_heads_workspace_bytes(rows, n_heads, d) bytes.
 * Returns HAWK_OK, HAWK_EINVAL (null pointer, shape not supported, workspace too small or
 * misaligned) or HAWK_EDEVICE. */
size_t hawk_spatial_heads_workspace_bytes(int rows, int n_heads, int d);
int hawk_spatial_heads(const float* h, const void* W_heads, const void* W_out, int rows, int n_heads, int d, int V_s,
                       float* q_logits, float* g_out, void* workspace, size_t workspace_bytes, void* stream);

/* Speculation cache: vertical predictions (rows of V_s logits) kept from the moment the position
 * they were made from is committed until raster order reaches the position they point to.  It
 * holds IW * VSD * (VSD + 1) / 2 entries, the size the method states: hawk_spec_cache_bytes is
 * that many rows of V_s floats plus one int32 tag per entry (rounded up to 256 bytes).
 * hawk_spec_cache_slot (host arithmetic only) is the entry a prediction of `depth` for position
 * `pos` waits in, -1 for bad arguments; entries that are outstanding at the same time never share
 * a slot.  hawk_spec_cache_reset marks every entry empty (once per image).
 * hawk_spec_cache_push: for r < rows with 0 <= pos[r] < IW * IH, the hidden state that predicted
 * position pos[r] gave q_vert[r * row_stride + (dep - 1) * V_s ...] as the logits for position
 * pos[r] + dep * IW, dep = 1..VSD; predictions for positions below the image are dropped, rows with
 * pos[r] out of range skipped (the rows of a verify pass that were not committed).  The positions
 * of one call are distinct, rows <= IW; row_stride (in floats) >= VSD * V_s. */
size_t hawk_spec_cache_bytes(int IW, int VSD, int V_s);
int hawk_spec_cache_slot(int IW, int VSD, int pos, int depth);
int hawk_spec_cache_reset(void* cache, int IW, int VSD, int V_s, void* stream);
int hawk_spec_cache_push(void* cache, int IW, int IH, int VSD, int V_s, const int32_t* pos, const float* q_vert,
                         size_t row_stride, int rows, void* stream);

/* Spatial sampling pool at the positions target[i], i < n: VertSpec(t) - the cached predictions
 * made from t - delta * IW with depth delta, delta = 1..VSD, those that exist, in ascending delta
 * - followed by the horizontal proposal q_horiz[i * horiz_stride ...] (the vertical candidate is
 * verified first, as in the appendix).  pool_logits [n][VSD + 1][V_s] receives the members'
 * logits packed to the front (rows beyond the count are left as they were), pool_m [n] the count,
 * pool_delta [n][VSD + 1] each member's delta (0 = horizontal, -1 = no member).  target[i] outside
 * 0 .. IW * IH - 1: count 0.  pool_logits, pool_m and pool_delta feed hawk_sample_rows (one
 * candidate per member) and hawk_multi_verify (q_logits, m_rows). */
int hawk_spec_pool(const void* cache, int IW, int IH, int VSD, int V_s, const int32_t* target, const float* q_horiz,
                   size_t horiz_stride, int n, float* pool_logits, int32_t* pool_m, int32_t* pool_delta, void* stream);

/* One draw per row from warp(logits[r]) by inverse CDF over ascending token index with u[r]
 * (warp as in hawk_multi_verify): the candidates of a pool.  logits [rows][n] fp32, n <= 16384;
 * skip (may be NULL) [rows]: rows with a negative entry are not read and give -1 (pass
 * pool_delta). */
int hawk_sample_rows(const float* logits, const int32_t* skip, const float* u, int rows, int n, float temperature,
                     int top_k, int32_t* out_token, void* stream);

/* The whole scheme over one image as one call (Method, overview figure and "Sampling and Verification"):
 * prefill; then, per pass: the dual-direction heads on the hidden states of the rows committed by the
 * pass before (hawk_spatial_heads; heads 0..HD-1 horizontal - head j for position T + j + 1 -, heads
 * HD..HD+VSD-1 vertical - depth 1..VSD), their vertical predictions into the speculation cache, the
 * sampling pools of the HD positions ahead (cached vertical predictions in ascending depth, then the
 * last row's horizontal proposal), one candidate per pool member (hawk_sample_rows), the target pass
 * over the candidate tree with its walk (hawk_verify_tree), commit of the accepted candidates and the
 * extra token.  When fewer positions are left than the widest tree has rows (1 + m + ... + m^HD, m = VSD
 * + 1), ordinary steps with one draft token of the context's own draft head finish the image.
 * One prompt (a context created for more can be used), no guidance (HAWK_EINVAL for a context created
 * with it); the context's k_max + 1 must be
 * at least the widest tree's rows; HD in 1..8, VSD in 0..7.
 * cond (host) [n_cond][d_model]; W_heads (DEVICE) [HD + VSD][d][d] bf16, W_out (DEVICE) [V_s][d] bf16 as for
 * hawk_spatial_heads; workspace (DEVICE, 256-byte aligned) of hawk_generate_spatial_workspace_bytes(cfg,
 * grid_w, HD, VSD) bytes (0: bad arguments), which holds the speculation cache and every intermediate.
 * Uniforms come from hawk_generate's counter-based generator with prompt 0 and step = pass number
 * (from 1; the ordinary steps at the end go on counting): slot 8 j + i draws the candidate of member i of
 * the pool at depth j + 1, slot 64 + 8 j + i is its acceptance test, slot 128 + j the draw after a
 * rejection at depth j + 1 (j = HD: the extra token after HD acceptances); step 0 slot 128 samples token
 * 0; an ordinary step uses slots 0, 64, 128 as in hawk_generate.
 * out_grid (host) [grid_h * grid_w] vocabulary ids; out_stats (host, may be NULL) [4]: tree passes,
 * candidates accepted in them, ordinary steps at the end, tokens.  The call synchronises once per pass
 * (the candidates and the walk's result come back to the host, which lays out the next pass).
 * Returns HAWK_OK or the first error of a step (HAWK_EINVAL, HAWK_ENOMEM for a workspace too small,
 * HAWK_ESTATE before hawk_load, HAWK_EDEVICE). */
size_t hawk_generate_spatial_workspace_bytes(const hawk_config* cfg, int grid_w, int HD, int VSD);
int hawk_generate_spatial(hawk_ctx* ctx, const float* cond, int n_cond, int grid_h, int grid_w, float temperature, int top_k,
                          const void* W_heads, const void* W_out, int HD, int VSD, uint64_t seed, void* workspace,
                          size_t workspace_bytes, int32_t* out_grid, int64_t* out_stats);

#ifdef __cplusplus
}
#endif
#endif
