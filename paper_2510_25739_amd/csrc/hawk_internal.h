// Internal declarations shared by the translation units of libhawk (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/hawk.h"

namespace hawk {

constexpr int kMaxK = 63;          // slots 0..63 of the uniform generator are draft slots
constexpr int kSlotDraft = 0, kSlotAcc = 64, kSlotFinal = 128;
constexpr int kSampThreads = 1024; // threads of one sampling workgroup

// Per-row result of the temperature/top-k warp: enough to re-evaluate the weight of any
// token of the row without repeating the selection.
struct WarpStat {
    double total;       // sum of the kept weights exp(z - zmax)
    float zmax;         // largest scaled logit
    uint32_t tau;       // order-preserving key of the smallest kept scaled logit
    int32_t tie_cut;    // entries equal to tau are kept up to and including this index
    int32_t onehot;     // >= 0: the row is the point mass on this index (greedy / replay)
};

// Where the uniforms of a step come from: host-supplied tables already copied to the
// device, or the counter-based generator.
struct UniformSrc {
    const float* draft;   // [B, k]
    const float* acc;     // [B, k]
    const float* fin;     // [B]
    uint64_t seed;
    const int32_t* step;  // device counter (generator mode)
    int32_t use_gen;
};

// Where draft tokens come from: 0 = sampled, 1 = the [B,k] table in the `forced` buffer,
// 2 = the replay grid at columns n + i - 1.
struct DraftMode {
    int32_t kind;
    int32_t point_mass;
};

// How the rows of a forward pass map to sequences and positions.
struct RowMap {
    int32_t mode;          // 0 = prefill (row r of sequence s at position r), 1 = step rows, 2 = tree rows
    int32_t rows_per_seq;  // C in prefill, k+1 in a step, nodes of the candidate tree
    int32_t n_seq, batch, n_cond;
    const int32_t* n;      // [B] committed tokens (step rows)
    const int32_t* k_eff;  // [B] drafts in flight, -1 = finished (step rows)
    // tree rows: row r is node r of the candidate tree (node 0 = the last committed token); its
    // position is that of the root plus its depth, its cache entry the root's plus r, and it attends
    // the committed entries, its ancestors (bit j of tree_anc[r]: node j) and itself
    const int32_t* tree_depth;            // [nodes]
    const unsigned long long* tree_anc;   // [nodes]
};

struct Offsets {  // byte offsets into the workspace
    size_t blob, kc, vc, n, k_eff, step, done, counters, grid, draft, forced, hprev, qstat, pstat;
    size_t x, a, qkv, o, u, din, g0, g1, ga, logit_s, logit_b, dlogit_s, dlogit_b;
    size_t u_draft, u_acc, u_fin, out_na, out_tok, inv_freq, replay, cond;
    size_t tree;    // candidate tree of a tree pass: int32 depth[64], then uint64 ancestors[64], then walk state
    size_t split;   // bf16 hi / lo planes of a GEMM input (batched shapes; 0: not present)
    size_t split2;  // second pair of planes: written by a GEMM's own epilogue while it reads the first
    size_t gpack;   // tile-major copy of the GEMM weights for the MFMA GEMM / GEMV kernels (0: not present)
    size_t total;
};

// Streaming (persistent-kernel) path: matrix kinds, workgroup count, workspace regions.
enum StreamKind { K_A = 0, K_C, K_D, K_E, K_LM, K_WD, K_NKIND };  // QKV, Wo, W1|W3, W2, output, draft
constexpr int kNWG = 256;  // persistent workgroups: one per compute unit
struct StreamOffsets { size_t wpack, tab, desc, arena, slot_bytes, bar, err, dbg, rope; };
struct StreamPlan;
// The same pass laid out on the chip's XCDs (xcd.hip): packed weights, job tables, tagged partial sums and
// sums of squares, per-XCD buffers, flag words.
struct XcdOffsets { size_t zero, wpack, desc, gtab, rtab, ptab, atab, xp, part[5], pss[5], xbuf, xcd_bytes, lflag, dbg, err, rope; };
struct XcdPlan;

struct Weights {  // byte offsets into the blob
    size_t E, g_f, W_out, W_d;
    size_t g1[128], Wqkv[128], Wo[128], g2[128], W13[128], W2[128];
};

}  // namespace hawk

struct hawk_ctx {
    hawk_config cfg;
    int L, d, H, hd, m, V, Vs, Smax, Bmax, Tmax, Nmax, Mmax, kmax;
    size_t esz, asz, ksz;  // bytes of a weight, an activation, a cache element
    uint8_t* ws;
    hipStream_t stream;
    hawk::Offsets off;
    hawk::Weights w;
    hawk::StreamOffsets soff;
    hawk::StreamPlan* plan;  // streaming path: job tables and barrier epoch (null until created)
    hawk::XcdOffsets xoff;
    hawk::XcdPlan* xplan;    // XCD-partitioned pass: plan and tag epoch (null until created)
    size_t err_off, rope_off;   // the persistent kernels' error word and rotary table [Tmax][hd / 2] (cos, sin) in the workspace
    int err_ready;           //   (set up by whichever plan exists; err_ready: the word is there and cleared)
    int dead;                // a persistent kernel gave up on a wait: its exchange state is undefined, every call fails
    int last_kernel;         // kernel of the last target pass: 0 one per operation, 1 grid-barrier kernel, 2 XCD-partitioned kernel
    size_t blob_bytes;
    size_t split_bytes;
    // matrices in the tile-major copy; pairs = m for W1|W3 stored with rows interleaved (W1 row f, W3 row f, ...)
    struct { size_t blob_off, pack_off; int N, K, pairs; } gpk[4 * 128 + 2];
    int n_gpk;
    size_t presplit_off;  // activation buffer whose bf16 planes are current (presplit_M rows of presplit_K), 0: none
    int presplit_M, presplit_K, presplit_buf;
    // per image
    int B, S, C, gh, gw, N, top_k, greedy;
    float temperature, inv_t, cfg_scale;
    int phase;   // 0 created, 1 loaded, 2 prefilled (draft next), 3 drafted (verify next)
    int k_last;
    int path;
    int launch_failed;
    int last_path;
    int stream_dbg;  // 1: the streaming kernel records per-phase timestamps
    void* pinned;  // small page-locked staging buffer for read-backs
    hipEvent_t ev[3];
    hipEvent_t* tev;  // event pool of hawk_run_steps phase timing
    size_t n_tev;
    hipEvent_t kev_a, kev_b;  // when set: recorded around the streaming kernel of the next target pass
    char err[256];
};

namespace hawk {

// fp32 -> bf16 hi (round to nearest even) and the bf16 remainder: v ~ hi + lo to about 16 bits
__device__ __forceinline__ void bf16_split(float v, unsigned& hi, unsigned& lo) {
    unsigned u = __float_as_uint(v);
    hi = (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
    u = __float_as_uint(v - __uint_as_float(hi << 16));
    lo = (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

template <typename T> inline T* wsp(hawk_ctx* c, size_t off) { return reinterpret_cast<T*>(c->ws + off); }

// ---- launchers implemented in generic.hip (dtype chosen from ctx->cfg.dtype) ----
void launch_embed_rows(hawk_ctx*, const RowMap&, int M);
void launch_cond_rows(hawk_ctx*, int M);                       // X <- condition vectors
// out[r] = rmsnorm(in[r * in_stride ...]) * gain, r < M (in_stride in elements)
// for_gemm: the next call is the GEMM that reads the output; its bf16 planes are written here too
void launch_rmsnorm(hawk_ctx*, size_t off_in, size_t in_stride, size_t off_gain, size_t off_out, int M,
                    bool for_gemm = false);
// Y[M][N] (+)= A[M][K] * W[N][K]^T ; out_f32: store fp32 (logits) instead of activations
void launch_gemm(hawk_ctx*, size_t off_a, int lda, size_t w_off, int N, int K, size_t off_y,
                 int ldy, int M, bool accumulate, bool out_f32);
// the same on the MFMA units (bf16, many rows); false if the shape is not covered (gemm.hip)
bool launch_gemm_mfma(hawk_ctx*, size_t off_a, int lda, size_t w_off, int N, int K, size_t off_y, int ldy, int M,
                      bool accumulate);
// A kernel that produces the input of the next GEMM (M rows of K values at off_a) can write that
// GEMM's bf16 hi / lo planes itself, [row][K] each: true and the planes if such a GEMM takes the
// MFMA path; the planes then count as current until the next launch_gemm call.
bool presplit_planes(hawk_ctx*, size_t off_a, int M, int K, uint16_t** hi, uint16_t** lo);
// fills the tile-major weight copy from the blob (after hawk_load's upload); 0 or -1
int gemm_pack_weights(hawk_ctx*);
void launch_rope_append(hawk_ctx*, const RowMap&, int layer, int M);
void launch_attention(hawk_ctx*, const RowMap&, int layer, int M);
// true: launch_attention also rotates q, k and appends k, v for these rows (no launch_rope_append)
bool attention_does_rope(const hawk_ctx*, const RowMap&);
// U[:, 0..m) = SiLU(A W1^T) * (A W3^T) in one MFMA kernel (and the bf16 planes of the result for the W2
// GEMM); false: not applicable, the caller runs the GEMM and launch_swiglu
bool launch_gemm_swiglu(hawk_ctx*, size_t off_a, int lda, size_t w13_off, int m, int K, size_t off_u, int M);
// Without a context: Y[M][N] = A W^T, A fp32 [M][K] (row stride lda), W bf16 row-major [N][K], on
// the MFMA kernels.  planes: room for 2 M K bf16 values (the two bf16 planes of A); A == nullptr:
// the planes are filled already (hi first, then lo).  false: the shape is not supported
// (K % 64, N % 16, lda % 4, ldy % 4).
bool gemm_rows_bf16(hipStream_t stream, const float* A, int lda, int M, int K, const uint16_t* W, int N, float* Y,
                    int ldy, uint16_t* planes);
// The draft heads' blocks in one launch (at most 16 rows, K % 128 == 0): W holds `blocks` square
// [K][K] matrices one after the other; G[(r * blocks + j)][K] = A[r] + silu(W_j A[r]) as fp32 and as
// the two bf16 planes the product that follows reads (planes_g: 2 M blocks K values; planes_a: 2 M K).
// false: shape not covered, the caller runs the product and the activation separately.
bool gemm_rows_heads(hipStream_t stream, const float* A, int M, int K, const uint16_t* W, int blocks, float* G,
                     uint16_t* planes_a, uint16_t* planes_g);
void launch_swiglu(hawk_ctx*, int M);
void launch_draft_input(hawk_ctx*, int i);                     // [g | E[left] | E[up]]
void launch_keep_hprev_prefill(hawk_ctx*);

// ---- streaming path, implemented in stream.hip ----
size_t stream_workspace(const hawk_ctx*, size_t base, StreamOffsets* out);  // extra workspace bytes
StreamPlan* stream_create(hawk_ctx*);     // plans the jobs, uploads tables (context has its workspace)
void stream_destroy(StreamPlan*);
void stream_plan_info(const hawk_ctx*, int64_t* out8);  // host-only summary of the plan
int stream_repack(hawk_ctx*);             // after the blob is on the device; 0 = ok
bool stream_ok(const hawk_ctx*, int k);   // can a step with k drafts run on the streaming path?
int launch_verify_stream(hawk_ctx*, int k);  // 0 = enqueued
bool stream_tree_ok(const hawk_ctx*, int n_nodes);   // can a pass over tree rows run on the streaming path?
int launch_verify_stream_tree(hawk_ctx*, int n_nodes, const int32_t* tree_depth, const unsigned long long* tree_anc);
bool stream_draft_ok(const hawk_ctx*);      // can draft micro-steps run on the streaming path?
int launch_draft_stream(hawk_ctx*, int i, size_t off_prev, size_t off_out);  // micro-step i up to its logits
int stream_error(hawk_ctx*);              // 1 if a wait of a persistent kernel timed out (synchronises)
bool stream_has_err_word(const hawk_ctx*);   // the persistent kernels' error word exists and is cleared

// ---- XCD-partitioned target pass, implemented in xcd.hip ----
size_t xcd_workspace(const hawk_ctx*, size_t base, XcdOffsets* out);   // extra workspace bytes (0: shape not covered)
XcdPlan* xcd_create(hawk_ctx*);           // plans the jobs, uploads tables, clears tags (context has its workspace)
void xcd_destroy(XcdPlan*);
int xcd_repack(hawk_ctx*);                // after the blob is on the device; 0 = ok
bool xcd_ok(const hawk_ctx*, int k);      // can a step with k drafts run on it?
int launch_verify_xcd(hawk_ctx*, int k, const int32_t* tree_depth = nullptr,
                      const unsigned long long* tree_anc = nullptr);   // the k + 1 step rows per sequence, or the k + 1 nodes of a candidate tree (device arrays)

// ---- launchers implemented in sampling.hip ----
void launch_plan(hawk_ctx*, int k);
void launch_first_token(hawk_ctx*, const UniformSrc&);
void launch_draft_sample(hawk_ctx*, int i, int k, const UniformSrc&, const DraftMode&);
void launch_verify_stats(hawk_ctx*, int k);
void launch_accept_commit(hawk_ctx*, int k, const UniformSrc&);
void launch_force_setup(hawk_ctx*, int cnt);
void launch_force_commit(hawk_ctx*, int cnt);
// multi-candidate verification of `rows` independent positions (device pointers); HAWK_* code
int launch_multi_verify(const float* p_logits, const float* q_logits, const int32_t* cand, const float* u_acc,
                        const float* u_final, const int32_t* m_rows, int rows, int m, int n, float temperature, int top_k,
                        int32_t* out_index, int32_t* out_token, double* out_resid, void* workspace,
                        size_t workspace_bytes, hipStream_t stream);
size_t multi_verify_workspace_bytes(int rows, int m);
int launch_multi_verify_static(const float* p_logits, const float* q_logits, const int32_t* cand, const float* u_acc,
                               const float* u_final, const int32_t* m_rows, int rows, int m, int n, float temperature,
                               int top_k, int32_t* out_index, int32_t* out_token, double* out_resid, hipStream_t stream);
int launch_sample_rows(const float* logits, const int32_t* skip, const float* u, int rows, int n, float temperature,
                       int top_k, int32_t* out_token, hipStream_t stream);

// ---- tree verification, implemented in tree.hip ----
constexpr int kTreeMaxDepth = 8;    // depths of a candidate tree
constexpr int kTreeMaxNodes = 64;   // nodes, the root included (one bit each in a row's ancestor mask)
// dst[r] = src[index[r]] (rows of n floats); uncond_shift > 0: guided with the row that many rows further on
void launch_gather_rows(hawk_ctx*, const float* src, const int32_t* index, float* dst, int rows, int n, int uncond_shift);
// one round of the walk (see tree_advance_kernel for the arrays)
void launch_tree_advance(hawk_ctx*, const int32_t* meta, int32_t* state, int32_t* path, int32_t* toks, int j);
// moves the accepted paths' cache entries into place, then commits tokens, n and the kept hidden state;
// acc [B] (-1: prompt not part of the pass), path [B][kTreeMaxDepth] node of the accepted candidate
// per depth, toks [B][kTreeMaxDepth + 1] vocabulary ids: device arrays
void launch_tree_commit(hawk_ctx*, const int32_t* acc, const int32_t* path, const int32_t* toks, int n_nodes);

// ---- spatial drafting structures, implemented in spatial.hip (no context; HAWK_* codes) ----
size_t spatial_heads_workspace_bytes(int rows, int n_heads, int d);
int launch_spatial_heads(const float* h, const uint16_t* W_heads, const uint16_t* W_out, int rows, int n_heads, int d,
                         int Vs, float* q_logits, float* g_out, void* workspace, size_t workspace_bytes,
                         hipStream_t stream);
size_t spec_cache_bytes(int IW, int VSD, int Vs);
int spec_cache_slot(int IW, int VSD, int pos, int depth);
int launch_spec_cache_reset(void* cache, int IW, int VSD, int Vs, hipStream_t stream);
int launch_spec_cache_push(void* cache, int IW, int IH, int VSD, int Vs, const int32_t* pos, const float* q_vert,
                           size_t row_stride, int rows, hipStream_t stream);
int launch_spec_pool(const void* cache, int IW, int IH, int VSD, int Vs, const int32_t* target, const float* q_horiz,
                     size_t horiz_stride, int n, float* pool_logits, int32_t* pool_m, int32_t* pool_delta,
                     hipStream_t stream);

}  // namespace hawk
