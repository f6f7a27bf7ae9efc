// Host side of libhawk: argument checking, workspace layout, and the order in which the
// kernels of a prefill / draft / verify / generate call are enqueued.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <new>

#include "hawk_internal.h"

#include <vector>

using namespace hawk;

namespace {

constexpr uint32_t kMagic = 0x4B574148u;
constexpr size_t kPinnedBytes = 1 << 20;

int fail(hawk_ctx* c, int code, const char* fmt, ...) __attribute__((format(printf, 3, 4)));
int fail(hawk_ctx* c, int code, const char* fmt, ...) {
    if (c) {
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(c->err, sizeof c->err, fmt, ap);
        va_end(ap);
    }
    return code;
}

#define HIP_TRY(c, call)                                                                     \
    do {                                                                                     \
        hipError_t e_ = (call);                                                              \
        if (e_ != hipSuccess) return fail((c), HAWK_EDEVICE, "%s: %s", #call, hipGetErrorString(e_)); \
    } while (0)

size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }

// Fills the derived dimensions; false if the configuration is invalid.
// The candidate tree of a tree step (Method, "Spatial Sampling Pool": Cartesian product of the
// per-position candidates): node 0 is the root, then depth by depth all combinations of the
// candidates so far, a node's children next to each other in candidate order.
struct TreeShape {
    int n_nodes, m_max;
    int first[kTreeMaxDepth + 2];               // first node of every depth; first[depth + 1] = n_nodes
    int depth[kTreeMaxNodes], parent[kTreeMaxNodes], digit[kTreeMaxNodes];   // digit: which candidate of its depth
    unsigned long long anc[kTreeMaxNodes];      // bit j: node j is an ancestor (the root included)
};
// 0 = ok, 1 = a depth without candidates (or too many), 2 = more nodes than max_nodes or 64
int tree_shape(int depth, const int32_t* m_depth, int max_nodes, TreeShape* t) {
    memset(t, 0, sizeof *t);
    t->n_nodes = 1;
    t->first[0] = 0;
    t->first[1] = 1;
    t->parent[0] = -1;
    for (int j = 0, width = 1; j < depth; ++j) {
        if (m_depth[j] < 1 || m_depth[j] > kTreeMaxNodes) return 1;
        width *= m_depth[j];
        t->n_nodes += width;
        if (t->n_nodes > kTreeMaxNodes || t->n_nodes > max_nodes) return 2;
        t->first[j + 2] = t->n_nodes;
        t->m_max = m_depth[j] > t->m_max ? m_depth[j] : t->m_max;
    }
    for (int j = 1; j <= depth; ++j)
        for (int i = t->first[j]; i < t->first[j + 1]; ++i) {
            const int idx = i - t->first[j];
            t->depth[i] = j;
            t->parent[i] = j == 1 ? 0 : t->first[j - 1] + idx / m_depth[j - 1];
            t->digit[i] = idx % m_depth[j - 1];
            t->anc[i] = t->anc[t->parent[i]] | (1ull << t->parent[i]);
        }
    return 0;
}

// Layout of the workspace region a tree step keeps its small arrays in (byte offsets from off.tree).
struct TreeArea {
    static constexpr size_t kCandCap = 512;   // depth x widest candidate list, per prompt
    static constexpr int kMetaFirst = 3, kMetaWidth = 16;   // meta: depth, nodes, m_max, first[10], ..., m_depth[8]
    enum { kCur = 0, kRows, kIdx, kTok, kWalking, kAcc, kStateWords };   // per-prompt words, [word][B]; kAcc last: acc, path, toks are contiguous
    size_t depth, anc, meta, state, path, toks, cand, u_acc, u_fin, bytes;
    explicit TreeArea(const hawk_ctx* c) : TreeArea((size_t)c->B) {}
    explicit TreeArea(size_t B) {
        depth = 0; anc = 256; meta = 768; state = 896;
        path = state + B * kStateWords * 4;
        toks = path + B * kTreeMaxDepth * 4;
        cand = (toks + B * (kTreeMaxDepth + 1) * 4 + 15) & ~(size_t)15;
        u_acc = cand + B * kCandCap * 4;
        u_fin = u_acc + B * kCandCap * 4;
        bytes = u_fin + B * (kTreeMaxDepth + 1) * 4;
    }
};

bool derive(const hawk_config* g, hawk_ctx* c) {
    if (!g) return false;
    if (g->n_layers < 1 || g->n_layers > 128 || g->d_model < 8 || g->d_model % 8 || g->n_heads < 1 ||
        g->d_model % g->n_heads || g->d_mlp < 8 || g->d_mlp % 8 || g->vocab < 1)
        return false;
    const int hd = g->d_model / g->n_heads;
    if (hd % 2 || hd > 256 || 256 % hd) return false;
    const int vs = g->samp_n ? g->samp_n : g->vocab;
    if (g->samp_lo < 0 || vs < 1 || (long long)g->samp_lo + vs > g->vocab) return false;
    if (g->max_cond < 1 || g->max_grid_h < 1 || g->max_grid_w < 1 || g->max_batch < 1 || g->max_batch > 1024 ||
        g->k_max < 0 || g->k_max > kMaxK)
        return false;
    if (g->dtype != HAWK_FP32 && g->dtype != HAWK_BF16) return false;
    if (!(g->rms_eps > 0.f) || !(g->rope_theta > 0.f) || (g->use_cfg != 0 && g->use_cfg != 1)) return false;
    c->cfg = *g;
    c->L = g->n_layers; c->d = g->d_model; c->H = g->n_heads; c->hd = hd; c->m = g->d_mlp; c->V = g->vocab;
    c->Vs = vs;
    c->Bmax = g->max_batch;
    c->Smax = g->max_batch * (g->use_cfg ? 2 : 1);
    c->Nmax = g->max_grid_h * g->max_grid_w;
    c->Tmax = g->max_cond + c->Nmax;
    c->kmax = g->k_max;
    const int rows = g->k_max + 1 > g->max_cond ? g->k_max + 1 : g->max_cond;
    c->Mmax = c->Smax * rows;
    c->esz = g->dtype == HAWK_FP32 ? 4 : 2;
    c->asz = g->dtype == HAWK_FP32 ? 8 : 4;
    c->ksz = g->dtype == HAWK_FP32 ? 8 : 2;
    // blob layout
    const size_t d = c->d, m = c->m, V = c->V, e = c->esz;
    size_t off = 64;
    c->w.E = off; off += V * d * e;
    for (int l = 0; l < c->L; ++l) {
        c->w.g1[l] = off; off += d * e;
        c->w.Wqkv[l] = off; off += 3 * d * d * e;
        c->w.Wo[l] = off; off += d * d * e;
        c->w.g2[l] = off; off += d * e;
        c->w.W13[l] = off; off += 2 * m * d * e;
        c->w.W2[l] = off; off += d * m * e;
    }
    c->w.g_f = off; off += d * e;
    c->w.W_out = off; off += V * d * e;
    c->w.W_d = off; off += 3 * d * d * e;
    c->blob_bytes = off;
    // workspace layout
    Offsets& o = c->off;
    size_t p = 0;
    auto take = [&](size_t bytes) { size_t at = p; p = align_up(p + bytes); return at; };
    const size_t B = c->Bmax, S = c->Smax, ks = c->kmax + 1, Vs = c->Vs, M = c->Mmax, a = c->asz;
    o.blob = take(c->blob_bytes);
    o.kc = take((size_t)c->L * S * c->Tmax * d * c->ksz);
    o.vc = take((size_t)c->L * S * c->Tmax * d * c->ksz);
    o.n = take(B * 4); o.k_eff = take(B * 4); o.step = take(4); o.done = take(4); o.counters = take(4 * 8);
    o.grid = take(B * c->Nmax * 4); o.draft = take(B * ks * 4); o.forced = take(B * ks * 4 + B * 4);
    o.hprev = take(S * d * a); o.qstat = take(B * ks * sizeof(WarpStat)); o.pstat = take(B * ks * sizeof(WarpStat));
    o.x = take(M * d * a); o.a = take(M * d * a); o.qkv = take(M * 3 * d * a); o.o = take(M * d * a);
    o.u = take(M * 2 * m * a); o.din = take(S * 3 * d * a); o.g0 = take(S * d * a); o.g1 = take(S * d * a);
    o.ga = take(S * d * a);
    o.logit_s = take(S * ks * Vs * 4); o.logit_b = take(B * ks * Vs * 4);
    o.dlogit_s = take(S * Vs * 4); o.dlogit_b = take(B * ks * Vs * 4);
    o.u_draft = take(B * ks * 4); o.u_acc = take(B * ks * 4); o.u_fin = take(B * 4);
    o.out_na = take(B * 4); o.out_tok = take(B * ks * 4); o.inv_freq = take((size_t)(hd / 2) * 8);
    o.replay = take(B * c->Nmax * 4); o.cond = take(S * (size_t)g->max_cond * d * 4);
    o.tree = take(TreeArea(B).bytes);
    const size_t widest = 3 * d > m ? 3 * d : m;
    c->split_bytes = g->dtype == HAWK_BF16 ? M * widest * 4 : 0;
    o.split = c->split_bytes ? take(c->split_bytes) : 0;
    o.split2 = c->split_bytes ? take(M * m * 4) : 0;
    // Tile-major copy of every GEMM weight (16 x 32 tiles, 1 KB each, in MFMA operand order): the
    // MFMA kernels then fetch whole kilobytes per request instead of 64-byte pieces of 16 rows.
    c->n_gpk = 0;
    o.gpack = 0;
    if (g->dtype == HAWK_BF16 && d % 32 == 0 && m % 32 == 0 && Vs % 16 == 0) {
        size_t q = 0;
        auto reg = [&](size_t blob_off, size_t N, size_t K, int pairs = 0) {
            auto& e2 = c->gpk[c->n_gpk++];
            e2.blob_off = blob_off; e2.pack_off = q; e2.N = (int)N; e2.K = (int)K; e2.pairs = pairs;
            q += N * K * 2;
        };
        for (int l = 0; l < c->L; ++l) {
            reg(c->w.Wqkv[l], 3 * d, d);
            reg(c->w.Wo[l], d, d);
            reg(c->w.W13[l], 2 * m, d, (int)m);   // W1 and W3 rows interleaved: SwiGLU in the GEMM's epilogue
            reg(c->w.W2[l], d, m);
        }
        reg(c->w.W_out + (size_t)g->samp_lo * d * e, Vs, d);
        reg(c->w.W_d, d, 3 * d);
        o.gpack = take(q);
    }
    p += stream_workspace(c, p, &c->soff);
    p += xcd_workspace(c, p, &c->xoff);
    o.total = p;
    return true;
}

RowMap step_map(hawk_ctx* c, int k) {
    RowMap m;
    m.mode = 1; m.rows_per_seq = k + 1; m.n_seq = c->S; m.batch = c->B; m.n_cond = c->C;
    m.n = wsp<int32_t>(c, c->off.n); m.k_eff = wsp<int32_t>(c, c->off.k_eff);
    m.tree_depth = nullptr; m.tree_anc = nullptr;
    return m;
}

// All decoder layers over M rows held in x (residual stream, updated in place).
void run_layers(hawk_ctx* c, const RowMap& map, int M) {
    const Offsets& o = c->off;
    const int d = c->d, m = c->m;
    for (int l = 0; l < c->L; ++l) {
        launch_rmsnorm(c, o.x, d, c->w.g1[l], o.a, M, true);
        launch_gemm(c, o.a, d, c->w.Wqkv[l], 3 * d, d, o.qkv, 3 * d, M, false, false);
        if (!attention_does_rope(c, map)) launch_rope_append(c, map, l, M);
        launch_attention(c, map, l, M);
        launch_gemm(c, o.o, d, c->w.Wo[l], d, d, o.x, d, M, true, false);
        launch_rmsnorm(c, o.x, d, c->w.g2[l], o.a, M, true);
        if (!launch_gemm_swiglu(c, o.a, d, c->w.W13[l], m, d, o.u, M)) {
            launch_gemm(c, o.a, d, c->w.W13[l], 2 * m, d, o.u, 2 * m, M, false, false);
            launch_swiglu(c, M);
        }
        launch_gemm(c, o.u, 2 * m, c->w.W2[l], d, m, o.x, d, M, true, false);
    }
}

size_t slice_off(const hawk_ctx* c) { return c->w.W_out + (size_t)c->cfg.samp_lo * c->d * c->esz; }

// Target pass over the step rows [last committed | drafts] and logits of every row.
void run_step_rows(hawk_ctx* c, int k) {
    const int M = c->S * (k + 1);
    RowMap map = step_map(c, k);
    launch_embed_rows(c, map, M);
    if (xcd_ok(c, k)) {  // one persistent kernel laid out on the XCDs: all layers and the output projection
        if (c->kev_a) (void)hipEventRecord(c->kev_a, c->stream);
        if (launch_verify_xcd(c, k) != 0) c->launch_failed = 1;
        if (c->kev_b) (void)hipEventRecord(c->kev_b, c->stream);
        c->last_path = 1;
        c->last_kernel = 2;
        return;
    }
    if (stream_ok(c, k)) {  // one persistent kernel: all layers and the output projection
        if (c->kev_a) (void)hipEventRecord(c->kev_a, c->stream);
        if (launch_verify_stream(c, k) != 0) c->launch_failed = 1;
        if (c->kev_b) (void)hipEventRecord(c->kev_b, c->stream);
        c->last_path = 1;
        c->last_kernel = 1;
        return;
    }
    c->last_path = 0;
    c->last_kernel = 0;
    run_layers(c, map, M);
    launch_rmsnorm(c, c->off.x, c->d, c->w.g_f, c->off.a, M, true);
    launch_gemm(c, c->off.a, c->d, slice_off(c), c->Vs, c->d, c->off.logit_s, c->Vs, M, false, true);
}

void enqueue_draft(hawk_ctx* c, int k, const UniformSrc& us, const DraftMode& dm) {
    launch_plan(c, k);
    for (int i = 1; i <= k; ++i) {
        const size_t g = (i & 1) ? c->off.g1 : c->off.g0;
        if (stream_draft_ok(c)) {  // one persistent kernel: W_d, final norm, output projection
            const size_t prev = (i == 1) ? c->off.hprev : (((i - 1) & 1) ? c->off.g1 : c->off.g0);
            if (launch_draft_stream(c, i, prev, g) != 0) c->launch_failed = 1;
            launch_draft_sample(c, i, k, us, dm);
            continue;
        }
        launch_draft_input(c, i);
        launch_gemm(c, c->off.din, 3 * c->d, c->w.W_d, c->d, 3 * c->d, g, c->d, c->S, false, false);
        launch_rmsnorm(c, g, c->d, c->w.g_f, c->off.ga, c->S);
        launch_gemm(c, c->off.ga, c->d, slice_off(c), c->Vs, c->d, c->off.dlogit_s, c->Vs, c->S, false, true);
        launch_draft_sample(c, i, k, us, dm);
    }
}

void enqueue_verify(hawk_ctx* c, int k, const UniformSrc& us) {
    run_step_rows(c, k);
    launch_verify_stats(c, k);
    launch_accept_commit(c, k, us);
}

int check_image_args(hawk_ctx* c, int batch, int n_cond, int grid_h, int grid_w, float temperature, int top_k,
                     float cfg_scale) {
    if (batch < 1 || batch > c->Bmax) return fail(c, HAWK_EINVAL, "batch %d outside [1, %d]", batch, c->Bmax);
    if (n_cond < 1 || n_cond > c->cfg.max_cond)
        return fail(c, HAWK_EINVAL, "n_cond %d outside [1, %d]", n_cond, c->cfg.max_cond);
    if (grid_h < 1 || grid_w < 1 || grid_h > c->cfg.max_grid_h || grid_w > c->cfg.max_grid_w)
        return fail(c, HAWK_EINVAL, "grid %dx%d outside the context's %dx%d", grid_h, grid_w, c->cfg.max_grid_h,
                    c->cfg.max_grid_w);
    if (!(temperature >= 0.f) || !isfinite(temperature)) return fail(c, HAWK_EINVAL, "temperature must be >= 0");
    if (top_k < 1 || top_k > c->Vs) return fail(c, HAWK_EINVAL, "top_k %d outside [1, %d]", top_k, c->Vs);
    if (c->cfg.use_cfg ? (cfg_scale == 1.0f) : (cfg_scale != 1.0f))
        return fail(c, HAWK_EINVAL, "cfg_scale %g does not match the context (use_cfg = %d)", (double)cfg_scale,
                    c->cfg.use_cfg);
    return HAWK_OK;
}

int enqueue_prefill(hawk_ctx* c, const float* cond, const float* uncond, int batch, int n_cond, int grid_h,
                    int grid_w, float temperature, int top_k, float cfg_scale, const UniformSrc& us) {
    c->B = batch; c->S = batch * (c->cfg.use_cfg ? 2 : 1); c->C = n_cond; c->gh = grid_h; c->gw = grid_w;
    c->N = grid_h * grid_w; c->temperature = temperature; c->top_k = top_k; c->cfg_scale = cfg_scale;
    c->greedy = (temperature == 0.f || top_k == 1) ? 1 : 0;
    c->inv_t = c->greedy ? 1.0f : 1.0f / temperature;
    const size_t per = (size_t)batch * n_cond * c->d * 4;
    HIP_TRY(c, hipMemsetAsync(c->ws + c->off.n, 0, c->off.grid - c->off.n, c->stream));
    HIP_TRY(c, hipMemcpyAsync(c->ws + c->off.cond, cond, per, hipMemcpyHostToDevice, c->stream));
    if (c->cfg.use_cfg)
        HIP_TRY(c, hipMemcpyAsync(c->ws + c->off.cond + per, uncond, per, hipMemcpyHostToDevice, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));  // the host buffers may be pageable
    const int M = c->S * n_cond;
    RowMap map;
    map.mode = 0; map.rows_per_seq = n_cond; map.n_seq = c->S; map.batch = c->B; map.n_cond = n_cond;
    map.n = nullptr; map.k_eff = nullptr; map.tree_depth = nullptr; map.tree_anc = nullptr;
    launch_cond_rows(c, M);
    run_layers(c, map, M);
    launch_keep_hprev_prefill(c);
    // final norm + output projection of the last condition row of every sequence
    launch_rmsnorm(c, c->off.x + (size_t)(n_cond - 1) * c->d * c->asz, (size_t)n_cond * c->d, c->w.g_f, c->off.a,
                   c->S);
    launch_gemm(c, c->off.a, c->d, slice_off(c), c->Vs, c->d, c->off.logit_s, c->Vs, c->S, false, true);
    launch_first_token(c, us);
    HIP_TRY(c, hipGetLastError());
    return HAWK_OK;
}

int upload(hawk_ctx* c, size_t off, const void* host, size_t bytes) {
    if (bytes == 0) return HAWK_OK;
    HIP_TRY(c, hipMemcpyAsync(c->ws + off, host, bytes, hipMemcpyHostToDevice, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    return HAWK_OK;
}

const char* const kDeadMsg =
    "a wait inside a persistent kernel timed out: the results of that step are invalid and the context's exchange "
    "buffers are in an undefined state - destroy the context and create a new one";

// Copies results to the host.  Every result a caller sees passes through here, so this is also where
// the persistent kernels' error word is read - in the same synchronisation as the data.
int download(hawk_ctx* c, void* host, size_t off, size_t bytes) {
    if (bytes == 0) return HAWK_OK;
    unsigned e = 0;
    HIP_TRY(c, hipMemcpyAsync(host, c->ws + off, bytes, hipMemcpyDeviceToHost, c->stream));
    if (stream_has_err_word(c)) HIP_TRY(c, hipMemcpyAsync(&e, c->ws + c->err_off, 4, hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    if (c->launch_failed) return fail(c, HAWK_EDEVICE, "launch of a persistent kernel failed");
    if (e != 0) {
        c->dead = 1;
        return fail(c, HAWK_EDEVICE, "%s", kDeadMsg);
    }
    return HAWK_OK;
}

// After a synchronisation: did a persistent kernel fail to launch or give up on a wait?
int check_stream(hawk_ctx* c) {
    if (c->launch_failed) return fail(c, HAWK_EDEVICE, "launch of a persistent kernel failed");
    if (stream_error(c)) {
        c->dead = 1;
        return fail(c, HAWK_EDEVICE, "%s", kDeadMsg);
    }
    return HAWK_OK;
}

// First line of every call that works on a context's state.
#define HAWK_LIVE(c)                                             \
    do {                                                         \
        if ((c)->dead) return fail((c), HAWK_EDEVICE, "%s", kDeadMsg); \
    } while (0)

bool uniforms_ok(const float* u, size_t n) {
    for (size_t i = 0; i < n; ++i)
        if (!(u[i] >= 0.f && u[i] < 1.f)) return false;
    return true;
}

}  // namespace

extern "C" {

size_t hawk_workspace_bytes(const hawk_config* cfg) {
    hawk_ctx tmp;
    memset(&tmp, 0, sizeof tmp);
    return derive(cfg, &tmp) ? tmp.off.total : 0;
}

int hawk_plan_info(const hawk_config* cfg, int64_t* out8) {
    if (!out8) return HAWK_EINVAL;
    hawk_ctx tmp;
    memset(&tmp, 0, sizeof tmp);
    if (!derive(cfg, &tmp)) return HAWK_EINVAL;
    stream_plan_info(&tmp, out8);
    return HAWK_OK;
}

int hawk_create(const hawk_config* cfg, void* workspace, size_t workspace_bytes, void* hip_stream, hawk_ctx** out) {
    if (!out) return HAWK_EINVAL;
    *out = nullptr;
    hawk_ctx* c = new (std::nothrow) hawk_ctx;
    if (!c) return HAWK_ENOMEM;
    memset(c, 0, sizeof *c);
    if (!derive(cfg, c)) { delete c; return HAWK_EINVAL; }
    if (!workspace || ((uintptr_t)workspace & 255)) { delete c; return HAWK_EINVAL; }
    if (workspace_bytes < c->off.total) { delete c; return HAWK_ENOMEM; }
    c->ws = static_cast<uint8_t*>(workspace);
    c->stream = static_cast<hipStream_t>(hip_stream);
    c->path = 1;
    c->last_path = -1;
    if (hipHostMalloc(&c->pinned, kPinnedBytes, hipHostMallocDefault) != hipSuccess) { delete c; return HAWK_EDEVICE; }
    for (int i = 0; i < 3; ++i)
        if (hipEventCreate(&c->ev[i]) != hipSuccess) { (void)hipHostFree(c->pinned); delete c; return HAWK_EDEVICE; }
    // rotary frequencies theta^(-2j/hd), computed once in double
    double* f = static_cast<double*>(c->pinned);
    for (int j = 0; j < c->hd / 2; ++j) f[j] = pow((double)c->cfg.rope_theta, -2.0 * j / (double)c->hd);
    if (hipMemcpyAsync(c->ws + c->off.inv_freq, f, (size_t)(c->hd / 2) * 8, hipMemcpyHostToDevice, c->stream) != hipSuccess ||
        hipStreamSynchronize(c->stream) != hipSuccess) {
        hawk_destroy(c);
        return HAWK_EDEVICE;
    }
    c->plan = stream_create(c);
    c->xplan = xcd_create(c);
    if (hipGetLastError() != hipSuccess || hipDeviceSynchronize() != hipSuccess) {
        hawk_destroy(c);
        return HAWK_EDEVICE;
    }
    *out = c;
    return HAWK_OK;
}

void hawk_destroy(hawk_ctx* c) {
    if (!c) return;
    (void)hipStreamSynchronize(c->stream);
    stream_destroy(c->plan);
    xcd_destroy(c->xplan);
    for (int i = 0; i < 3; ++i)
        if (c->ev[i]) (void)hipEventDestroy(c->ev[i]);
    if (c->pinned) (void)hipHostFree(c->pinned);
    for (size_t i = 0; i < c->n_tev; ++i) (void)hipEventDestroy(c->tev[i]);
    free(c->tev);
    delete c;
}

const char* hawk_last_error(const hawk_ctx* c) { return c ? c->err : "null context"; }

int hawk_set_path(hawk_ctx* c, int path) {
    if (!c) return HAWK_EINVAL;
    if (path < 0 || path > 2) return fail(c, HAWK_EINVAL, "path must be 0, 1 or 2");
    c->path = path;
    return HAWK_OK;
}

int hawk_last_path(const hawk_ctx* c) { return c ? c->last_path : -1; }

int hawk_last_kernel(const hawk_ctx* c) { return c ? c->last_kernel : -1; }

int hawk_debug_raise_timeout(hawk_ctx* c) {
    if (!c) return HAWK_EINVAL;
    if (!stream_has_err_word(c)) return fail(c, HAWK_ESTATE, "this context has no persistent-kernel plan");
    const unsigned one = 1;
    HIP_TRY(c, hipMemcpyAsync(c->ws + c->err_off, &one, 4, hipMemcpyHostToDevice, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    return HAWK_OK;
}

int hawk_phase_trace(hawk_ctx* c, int enable, uint64_t* out, size_t n_words) {
    if (!c) return HAWK_EINVAL;
    c->stream_dbg = enable ? 1 : 0;
    if (out && c->xplan && c->last_kernel == 2) {   // the XCD-partitioned kernel's stamps: [2 workgroups][512 stages][16]
        if (n_words > 2 * 512 * 16) n_words = 2 * 512 * 16;
        return download(c, out, c->xoff.dbg, n_words * 8);
    }
    if (out && c->plan) {
        if (n_words > 4 * 4096 * 8 + 2 * 256 * 256) n_words = 4 * 4096 * 8 + 2 * 256 * 256;
        return download(c, out, c->soff.dbg, n_words * 8);
    }
    return HAWK_OK;
}

size_t hawk_multi_verify_workspace_bytes(int rows, int m) {
    return rows > 0 && m > 0 ? hawk::multi_verify_workspace_bytes(rows, m) : 0;
}

int hawk_multi_verify(const float* p_logits, const float* q_logits, const int32_t* cand, const float* u_acc,
                      const float* u_final, const int32_t* m_rows, int rows, int m, int n, float temperature, int top_k,
                      int32_t* out_index, int32_t* out_token, double* out_resid, void* workspace,
                      size_t workspace_bytes, void* stream) {
    if (!p_logits || !q_logits || !cand || !u_acc || !u_final || !out_index || !out_token) return HAWK_EINVAL;
    if (rows < 0 || m < 1 || n < 1 || top_k < 1 || !(temperature >= 0.0f)) return HAWK_EINVAL;
    if (rows == 0) return HAWK_OK;
    return hawk::launch_multi_verify(p_logits, q_logits, cand, u_acc, u_final, m_rows, rows, m, n, temperature, top_k,
                                     out_index, out_token, out_resid, workspace, workspace_bytes,
                                     static_cast<hipStream_t>(stream));
}

int hawk_multi_verify_static(const float* p_logits, const float* q_logits, const int32_t* cand, const float* u_acc,
                             const float* u_final, const int32_t* m_rows, int rows, int m, int n, float temperature,
                             int top_k, int32_t* out_index, int32_t* out_token, double* out_resid, void* stream) {
    if (!p_logits || !q_logits || !cand || !u_acc || !u_final || !out_index || !out_token) return HAWK_EINVAL;
    if (rows < 0 || m < 1 || n < 1 || top_k < 1 || !(temperature >= 0.0f)) return HAWK_EINVAL;
    if (rows == 0) return HAWK_OK;
    return hawk::launch_multi_verify_static(p_logits, q_logits, cand, u_acc, u_final, m_rows, rows, m, n, temperature,
                                            top_k, out_index, out_token, out_resid, static_cast<hipStream_t>(stream));
}

size_t hawk_spatial_heads_workspace_bytes(int rows, int n_heads, int d) {
    return rows > 0 && n_heads > 0 && d > 0 ? hawk::spatial_heads_workspace_bytes(rows, n_heads, d) : 0;
}

int hawk_spatial_heads(const float* h, const void* W_heads, const void* W_out, int rows, int n_heads, int d, int V_s,
                       float* q_logits, float* g_out, void* workspace, size_t workspace_bytes, void* stream) {
    if (!h || !W_heads || !W_out || !q_logits) return HAWK_EINVAL;
    if (rows < 0 || n_heads < 1 || d < 1 || V_s < 1 || (long)rows * n_heads > 65535) return HAWK_EINVAL;
    if (rows == 0) return HAWK_OK;
    return hawk::launch_spatial_heads(h, static_cast<const uint16_t*>(W_heads), static_cast<const uint16_t*>(W_out), rows,
                                      n_heads, d, V_s, q_logits, g_out, workspace, workspace_bytes,
                                      static_cast<hipStream_t>(stream));
}

size_t hawk_spec_cache_bytes(int IW, int VSD, int V_s) {
    return IW > 0 && VSD > 0 && VSD <= 16 && V_s > 0 ? hawk::spec_cache_bytes(IW, VSD, V_s) : 0;
}

int hawk_spec_cache_slot(int IW, int VSD, int pos, int depth) { return hawk::spec_cache_slot(IW, VSD, pos, depth); }

int hawk_spec_cache_reset(void* cache, int IW, int VSD, int V_s, void* stream) {
    return hawk::launch_spec_cache_reset(cache, IW, VSD, V_s, static_cast<hipStream_t>(stream));
}

int hawk_spec_cache_push(void* cache, int IW, int IH, int VSD, int V_s, const int32_t* pos, const float* q_vert,
                         size_t row_stride, int rows, void* stream) {
    return hawk::launch_spec_cache_push(cache, IW, IH, VSD, V_s, pos, q_vert, row_stride, rows,
                                        static_cast<hipStream_t>(stream));
}

int hawk_spec_pool(const void* cache, int IW, int IH, int VSD, int V_s, const int32_t* target, const float* q_horiz,
                   size_t horiz_stride, int n, float* pool_logits, int32_t* pool_m, int32_t* pool_delta, void* stream) {
    return hawk::launch_spec_pool(cache, IW, IH, VSD, V_s, target, q_horiz, horiz_stride, n, pool_logits, pool_m,
                                  pool_delta, static_cast<hipStream_t>(stream));
}

int hawk_sample_rows(const float* logits, const int32_t* skip, const float* u, int rows, int n, float temperature,
                     int top_k, int32_t* out_token, void* stream) {
    if (!logits || !u || !out_token) return HAWK_EINVAL;
    if (rows < 0 || n < 1 || top_k < 1 || !(temperature >= 0.0f)) return HAWK_EINVAL;
    if (rows == 0) return HAWK_OK;
    return hawk::launch_sample_rows(logits, skip, u, rows, n, temperature, top_k, out_token,
                                    static_cast<hipStream_t>(stream));
}

int hawk_load(hawk_ctx* c, const void* host_blob, size_t nbytes) {
    if (!c) return HAWK_EINVAL;
    HAWK_LIVE(c);
    if (!host_blob) return fail(c, HAWK_EINVAL, "null blob");
    if (nbytes != c->blob_bytes)
        return fail(c, HAWK_EINVAL, "blob has %zu bytes, configuration needs %zu", nbytes, c->blob_bytes);
    const int32_t* h = static_cast<const int32_t*>(host_blob);
    if ((uint32_t)h[0] != kMagic || h[1] != 1) return fail(c, HAWK_EINVAL, "bad blob magic or version");
    if (h[2] != c->cfg.dtype || h[3] != c->L || h[4] != c->d || h[5] != c->H || h[6] != c->m || h[7] != c->V)
        return fail(c, HAWK_EINVAL, "blob header does not match the context's configuration");
    HIP_TRY(c, hipMemcpy(c->ws + c->off.blob, host_blob, nbytes, hipMemcpyHostToDevice));
    if (stream_repack(c) != 0) return fail(c, HAWK_EDEVICE, "re-tiling the weights for the streaming path failed");
    if (xcd_repack(c) != 0) return fail(c, HAWK_EDEVICE, "re-tiling the weights for the XCD-partitioned pass failed");
    if (gemm_pack_weights(c) != 0) return fail(c, HAWK_EDEVICE, "re-tiling the weights for the MFMA GEMMs failed");
    c->phase = 1;
    return HAWK_OK;
}

int hawk_prefill(hawk_ctx* c, const float* cond, const float* uncond, int batch, int n_cond, int grid_h, int grid_w,
                 float temperature, int top_k, float cfg_scale, const float* u_first) {
    if (!c) return HAWK_EINVAL;
    HAWK_LIVE(c);
    if (c->phase < 1) return fail(c, HAWK_ESTATE, "hawk_prefill before hawk_load");
    if (!cond || !u_first || (c->cfg.use_cfg && !uncond)) return fail(c, HAWK_EINVAL, "null input");
    int rc = check_image_args(c, batch, n_cond, grid_h, grid_w, temperature, top_k, cfg_scale);
    if (rc) return rc;
    if (!uniforms_ok(u_first, batch)) return fail(c, HAWK_EINVAL, "uniforms must lie in [0, 1)");
    rc = upload(c, c->off.u_fin, u_first, (size_t)batch * 4);
    if (rc) return rc;
    UniformSrc us;
    memset(&us, 0, sizeof us);
    us.fin = wsp<float>(c, c->off.u_fin);
    rc = enqueue_prefill(c, cond, uncond, batch, n_cond, grid_h, grid_w, temperature, top_k, cfg_scale, us);
    if (rc) return rc;
    c->phase = 2;
    return HAWK_OK;
}

int hawk_draft(hawk_ctx* c, int k, const float* u_draft, int32_t* out_draft) {
    if (!c) return HAWK_EINVAL;
    HAWK_LIVE(c);
    if (c->phase != 2 && c->phase != 3) return fail(c, HAWK_ESTATE, "hawk_draft needs a prefilled context");
    if (k < 0 || k > c->kmax || k > c->gw)
        return fail(c, HAWK_EINVAL, "k = %d outside [0, min(k_max = %d, grid_w = %d)]", k, c->kmax, c->gw);
    if (k > 0 && !u_draft) return fail(c, HAWK_EINVAL, "null uniforms");
    if (k > 0 && !uniforms_ok(u_draft, (size_t)c->B * k)) return fail(c, HAWK_EINVAL, "uniforms must lie in [0, 1)");
    int rc = upload(c, c->off.u_draft, u_draft, (size_t)c->B * k * 4);
    if (rc) return rc;
    UniformSrc us;
    memset(&us, 0, sizeof us);
    us.draft = wsp<float>(c, c->off.u_draft);
    DraftMode dm = {0, 0};
    enqueue_draft(c, k, us, dm);
    HIP_TRY(c, hipGetLastError());
    c->k_last = k;
    c->phase = 3;
    if (out_draft && k > 0) {
        int32_t* tmp = static_cast<int32_t*>(c->pinned);
        rc = download(c, tmp, c->off.draft, (size_t)c->B * (c->kmax + 1) * 4);
        if (rc) return rc;
        for (int b = 0; b < c->B; ++b)
            for (int i = 0; i < k; ++i) out_draft[b * k + i] = tmp[b * (c->kmax + 1) + i];
    }
    return HAWK_OK;
}

int hawk_draft_forced(hawk_ctx* c, int k, const int32_t* tokens, int point_mass) {
    if (!c) return HAWK_EINVAL;
    HAWK_LIVE(c);
    if (c->phase != 2 && c->phase != 3) return fail(c, HAWK_ESTATE, "hawk_draft_forced needs a prefilled context");
    if (k < 0 || k > c->kmax || k > c->gw)
        return fail(c, HAWK_EINVAL, "k = %d outside [0, min(k_max = %d, grid_w = %d)]", k, c->kmax, c->gw);
    if (k > 0 && !tokens) return fail(c, HAWK_EINVAL, "null tokens");
    for (size_t i = 0; i < (size_t)c->B * k; ++i)
        if (tokens[i] < c->cfg.samp_lo || tokens[i] >= c->cfg.samp_lo + c->Vs)
            return fail(c, HAWK_EINVAL, "forced token %d outside the sampled slice", tokens[i]);
    int rc = upload(c, c->off.forced, tokens, (size_t)c->B * k * 4);
    if (rc) return rc;
    UniformSrc us;
    memset(&us, 0, sizeof us);
    DraftMode dm = {1, point_mass ? 1 : 0};
    enqueue_draft(c, k, us, dm);
    HIP_TRY(c, hipGetLastError());
    HIP_TRY(c, hipStreamSynchronize(c->stream));  // the staging buffer may be reused by the next call
    c->k_last = k;
    c->phase = 3;
    return HAWK_OK;
}

int hawk_verify(hawk_ctx* c, int k, const float* u_acc, const float* u_final, int32_t* out_n_accept,
                int32_t* out_tokens) {
    if (!c) return HAWK_EINVAL;
    HAWK_LIVE(c);
    if (c->phase != 3 || k != c->k_last) return fail(c, HAWK_ESTATE, "hawk_verify(k) must follow hawk_draft(k)");
    if (!u_final || (k > 0 && !u_acc)) return fail(c, HAWK_EINVAL, "null uniforms");
    if (!uniforms_ok(u_final, c->B) || (k > 0 && !uniforms_ok(u_acc, (size_t)c->B * k)))
        return fail(c, HAWK_EINVAL, "uniforms must lie in [0, 1)");
    int rc = upload(c, c->off.u_acc, u_acc, (size_t)c->B * k * 4);
    if (!rc) rc = upload(c, c->off.u_fin, u_final, (size_t)c->B * 4);
    if (rc) return rc;
    UniformSrc us;
    memset(&us, 0, sizeof us);
    us.acc = wsp<float>(c, c->off.u_acc);
    us.fin = wsp<float>(c, c->off.u_fin);
    enqueue_verify(c, k, us);
    HIP_TRY(c, hipGetLastError());
    c->phase = 2;
    if (out_n_accept) {
        rc = download(c, out_n_accept, c->off.out_na, (size_t)c->B * 4);
        if (rc) return rc;
    }
    if (out_tokens) {
        rc = download(c, out_tokens, c->off.out_tok, (size_t)c->B * (k + 1) * 4);
        if (rc) return rc;
    }
    if (out_n_accept || out_tokens) return check_stream(c);
    return HAWK_OK;
}

int hawk_tree_layout(int depth, const int32_t* m_depth, int32_t* out_parent, int32_t* out_depth, int32_t* out_candidate,
                     uint64_t* out_ancestors) {
    if (!m_depth || depth < 1 || depth > kTreeMaxDepth) return -1;
    TreeShape ts;
    if (tree_shape(depth, m_depth, kTreeMaxNodes, &ts) != 0) return -1;
    for (int i = 0; i < ts.n_nodes; ++i) {
        if (out_parent) out_parent[i] = ts.parent[i];
        if (out_depth) out_depth[i] = ts.depth[i];
        if (out_candidate) out_candidate[i] = i ? ts.digit[i] : -1;
        if (out_ancestors) out_ancestors[i] = ts.anc[i];
    }
    return ts.n_nodes;
}

int hawk_verify_tree(hawk_ctx* c, int depth, const int32_t* m_depth, const int32_t* cand, const float* q_logits,
                     const float* u_acc, const float* u_final, int32_t* out_n_accept, int32_t* out_tokens) {
    if (!c) return HAWK_EINVAL;
    HAWK_LIVE(c);
    if (c->phase < 2) return fail(c, HAWK_ESTATE, "hawk_verify_tree before hawk_prefill");
    if (!m_depth || !cand || !q_logits || !u_acc || !u_final) return fail(c, HAWK_EINVAL, "null input");
    if (depth < 1 || depth > kTreeMaxDepth) return fail(c, HAWK_EINVAL, "depth = %d outside [1, %d]", depth, kTreeMaxDepth);
    const int B = c->B;
    TreeShape ts;
    const int shape_rc = tree_shape(depth, m_depth, c->kmax + 1, &ts);
    if (shape_rc == 1) return fail(c, HAWK_EINVAL, "every depth needs between 1 and %d candidates", kTreeMaxNodes);
    if (shape_rc == 2)
        return fail(c, HAWK_EINVAL, "the tree has more than %d nodes (64, or k_max + 1 rows per sequence)",
                    c->kmax + 1 < kTreeMaxNodes ? c->kmax + 1 : kTreeMaxNodes);
    const int m_max = ts.m_max, n_nodes = ts.n_nodes;
    const int* first = ts.first;
    if (c->Vs > 16384) return fail(c, HAWK_EINVAL, "sampled slice beyond 16384 entries");
    for (size_t i = 0; i < (size_t)depth * B * m_max; ++i) {
        const int j = (int)(i / ((size_t)B * m_max)), slot = (int)(i % m_max);
        if (slot < m_depth[j] && (cand[i] < 0 || cand[i] >= c->Vs)) return fail(c, HAWK_EINVAL, "candidate outside the sampled slice");
        if (slot < m_depth[j] && !(u_acc[i] >= 0.f && u_acc[i] < 1.f)) return fail(c, HAWK_EINVAL, "uniforms must lie in [0, 1)");
    }
    if (!uniforms_ok(u_final, (size_t)(depth + 1) * B)) return fail(c, HAWK_EINVAL, "uniforms must lie in [0, 1)");
    int32_t n_now[256];
    if (B > 256) return fail(c, HAWK_EINVAL, "batch beyond 256");
    int rc = download(c, n_now, c->off.n, (size_t)B * 4);
    if (rc) return rc;
    bool any = false;
    for (int b = 0; b < B; ++b) {
        if (n_now[b] >= c->N) continue;   // finished
        if (n_now[b] + n_nodes > c->N)
            return fail(c, HAWK_EINVAL, "prompt %d: %d tokens left, the tree needs room for %d rows (use hawk_verify near the end)",
                        b, c->N - n_now[b], n_nodes);
        any = true;
    }
    // host image of everything the device needs, staged in page-locked memory and sent in one go
    const int ks = c->kmax + 1;
    const TreeArea ta(c);
    if ((size_t)depth * m_max > TreeArea::kCandCap) return fail(c, HAWK_EINVAL, "depth x widest candidate list beyond %d", (int)TreeArea::kCandCap);
    char* stage = static_cast<char*>(c->pinned);
    const size_t tok_at = (ta.bytes + 255) & ~(size_t)255, keff_at = tok_at + (((size_t)B * ks * 4 + 255) & ~(size_t)255);
    if (keff_at + (size_t)B * 4 > kPinnedBytes) return fail(c, HAWK_EINVAL, "batch too large for the staging buffer");
    memset(stage, 0, keff_at + (size_t)B * 4);
    int32_t* node_depth = reinterpret_cast<int32_t*>(stage + ta.depth);
    unsigned long long* anc = reinterpret_cast<unsigned long long*>(stage + ta.anc);
    int32_t* meta = reinterpret_cast<int32_t*>(stage + ta.meta);
    int32_t* tokens = reinterpret_cast<int32_t*>(stage + tok_at);
    int32_t* keff = reinterpret_cast<int32_t*>(stage + keff_at);
    for (int i = 0; i < n_nodes; ++i) {
        node_depth[i] = ts.depth[i];
        anc[i] = ts.anc[i];
    }
    const int* digit = ts.digit;
    meta[0] = depth; meta[1] = n_nodes; meta[2] = m_max;
    for (int j = 0; j <= depth + 1; ++j) meta[TreeArea::kMetaFirst + j] = first[j];
    for (int j = 0; j < depth; ++j) meta[TreeArea::kMetaWidth + j] = m_depth[j];
    int spare = -1;   // a row with valid logits for prompts that take no part (their results are ignored)
    for (int b = 0; b < B; ++b)
        if (n_now[b] < c->N && spare < 0) spare = b * n_nodes;
    int32_t* st = reinterpret_cast<int32_t*>(stage + ta.state);
    for (int b = 0; b < B; ++b) {
        const bool on = n_now[b] < c->N;
        keff[b] = on ? n_nodes - 1 : -1;
        for (int i = 0; i < ks; ++i) tokens[(size_t)b * ks + i] = -1;
        for (int i = 1; i < n_nodes; ++i)
            tokens[(size_t)b * ks + i - 1] = c->cfg.samp_lo + cand[((size_t)(node_depth[i] - 1) * B + b) * m_max + digit[i]];
        st[TreeArea::kCur * B + b] = on ? b * n_nodes : (spare < 0 ? 0 : spare);
        st[TreeArea::kRows * B + b] = on ? m_depth[0] : 0;
        st[TreeArea::kAcc * B + b] = on ? 0 : -1;
        st[TreeArea::kWalking * B + b] = on ? 1 : 0;
    }
    int32_t* toks_img = reinterpret_cast<int32_t*>(stage + ta.toks);
    for (size_t i = 0; i < (size_t)B * (kTreeMaxDepth + 1); ++i) toks_img[i] = -1;
    memcpy(stage + ta.cand, cand, (size_t)depth * B * m_max * 4);
    memcpy(stage + ta.u_acc, u_acc, (size_t)depth * B * m_max * 4);
    memcpy(stage + ta.u_fin, u_final, (size_t)(depth + 1) * B * 4);
    if (any) {
        HIP_TRY(c, hipMemcpyAsync(c->ws + c->off.tree, stage, ta.bytes, hipMemcpyHostToDevice, c->stream));
        HIP_TRY(c, hipMemcpyAsync(c->ws + c->off.draft, tokens, (size_t)B * ks * 4, hipMemcpyHostToDevice, c->stream));
        HIP_TRY(c, hipMemcpyAsync(c->ws + c->off.k_eff, keff, (size_t)B * 4, hipMemcpyHostToDevice, c->stream));
        // the target pass over all nodes
        const size_t t0 = c->off.tree;
        RowMap map = step_map(c, n_nodes - 1);
        map.mode = 2;
        map.tree_depth = wsp<int32_t>(c, t0 + ta.depth);
        map.tree_anc = wsp<unsigned long long>(c, t0 + ta.anc);
        const int M = c->S * n_nodes;
        c->presplit_off = 0;
        launch_embed_rows(c, map, M);
        if (xcd_ok(c, n_nodes - 1)) {       // one persistent kernel, laid out on the XCDs: all layers and the output projection
            if (launch_verify_xcd(c, n_nodes - 1, map.tree_depth, map.tree_anc) != 0) c->launch_failed = 1;
            c->last_path = 1;
            c->last_kernel = 2;
        } else if (stream_tree_ok(c, n_nodes)) {   // the same with grid barriers
            if (launch_verify_stream_tree(c, n_nodes, map.tree_depth, map.tree_anc) != 0) c->launch_failed = 1;
            c->last_path = 1;
            c->last_kernel = 1;
        } else {                            // one kernel per operation
            c->last_path = 0;
            c->last_kernel = 0;
            run_layers(c, map, M);
            launch_rmsnorm(c, c->off.x, c->d, c->w.g_f, c->off.a, M, true);
            launch_gemm(c, c->off.a, c->d, slice_off(c), c->Vs, c->d, c->off.logit_s, c->Vs, M, false, true);
        }
        HIP_TRY(c, hipGetLastError());
        // The walk, on the device: per depth, the row of the node each prompt stands on is gathered as
        // the target of that depth's candidates, verified, and a small kernel moves the prompt to the
        // accepted child or ends its walk.  All depth + 1 rounds are enqueued; prompts that have
        // stopped take part with no candidates and their results are ignored.
        int32_t* dstate = wsp<int32_t>(c, t0 + ta.state);
        float* p_rows = wsp<float>(c, c->off.logit_b);
        for (int j = 0; j <= depth; ++j) {
            launch_gather_rows(c, wsp<float>(c, c->off.logit_s), dstate + TreeArea::kCur * B, p_rows, B, c->Vs,
                               c->cfg.use_cfg ? B * n_nodes : 0);
            const int m_call = j < depth ? m_max : 1;
            rc = launch_multi_verify(p_rows, j < depth ? q_logits + (size_t)j * B * m_max * c->Vs : p_rows,
                                     wsp<int32_t>(c, t0 + ta.cand) + (j < depth ? (size_t)j * B * m_max : 0),
                                     wsp<float>(c, t0 + ta.u_acc) + (j < depth ? (size_t)j * B * m_max : 0),
                                     wsp<float>(c, t0 + ta.u_fin) + (size_t)j * B, dstate + TreeArea::kRows * B, B, m_call,
                                     c->Vs, c->temperature, c->top_k, dstate + TreeArea::kIdx * B, dstate + TreeArea::kTok * B,
                                     nullptr, wsp<void>(c, c->off.qstat), 2 * (size_t)B * ks * sizeof(WarpStat), c->stream);
            if (rc) return fail(c, rc, "launch of the verification kernel failed");
            launch_tree_advance(c, wsp<int32_t>(c, t0 + ta.meta), dstate, wsp<int32_t>(c, t0 + ta.path),
                                wsp<int32_t>(c, t0 + ta.toks), j);
        }
        launch_tree_commit(c, dstate + TreeArea::kAcc * B, wsp<int32_t>(c, t0 + ta.path), wsp<int32_t>(c, t0 + ta.toks), n_nodes);
        HIP_TRY(c, hipGetLastError());
        // acc, path and tokens come back in one copy (they are contiguous)
        HIP_TRY(c, hipMemcpyAsync(stage + ta.state, c->ws + t0 + ta.state, ta.cand - ta.state, hipMemcpyDeviceToHost, c->stream));
        HIP_TRY(c, hipStreamSynchronize(c->stream));
        rc = check_stream(c);
        if (rc) return rc;
    }
    c->phase = 2;
    for (int b = 0; b < B; ++b) {
        const int a = st[TreeArea::kAcc * B + b];
        if (out_n_accept) out_n_accept[b] = a;
        if (out_tokens)
            for (int i = 0; i <= depth; ++i)
                out_tokens[(size_t)b * (depth + 1) + i] = a >= 0 && i <= a ? toks_img[(size_t)b * (kTreeMaxDepth + 1) + i] : -1;
    }
    return HAWK_OK;
}

int hawk_force(hawk_ctx* c, const int32_t* n_from, const int32_t* tokens, int cnt) {
    if (!c) return HAWK_EINVAL;
    HAWK_LIVE(c);
    if (c->phase < 2) return fail(c, HAWK_ESTATE, "hawk_force before hawk_prefill");
    if (!n_from || !tokens) return fail(c, HAWK_EINVAL, "null input");
    if (cnt < 1 || cnt > c->kmax + 1) return fail(c, HAWK_EINVAL, "cnt = %d outside [1, k_max + 1]", cnt);
    int32_t* cur = static_cast<int32_t*>(c->pinned);
    int rc = download(c, cur, c->off.n, (size_t)c->B * 4);
    if (rc) return rc;
    for (int b = 0; b < c->B; ++b) {
        if (n_from[b] < 1 || n_from[b] > cur[b] || n_from[b] + cnt > c->N)
            return fail(c, HAWK_EINVAL, "n_from[%d] = %d invalid (current n = %d, N = %d, cnt = %d)", b, n_from[b],
                        cur[b], c->N, cnt);
        for (int i = 0; i < cnt; ++i)
            if (tokens[b * cnt + i] < 0 || tokens[b * cnt + i] >= c->V)
                return fail(c, HAWK_EINVAL, "token outside the vocabulary");
    }
    rc = upload(c, c->off.forced, tokens, (size_t)c->B * cnt * 4);
    if (!rc) rc = upload(c, c->off.u_draft, n_from, (size_t)c->B * 4);  // staged in the draft-uniform slot
    if (rc) return rc;
    launch_force_setup(c, cnt);
    run_step_rows(c, cnt - 1);
    launch_verify_stats(c, cnt - 1);
    launch_force_commit(c, cnt);
    HIP_TRY(c, hipGetLastError());
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    c->phase = 2;
    return check_stream(c);
}

int hawk_generate(hawk_ctx* c, const float* cond, const float* uncond, int batch, int n_cond, int grid_h, int grid_w,
                  int k, float temperature, int top_k, float cfg_scale, uint64_t seed, const int32_t* replay_tokens,
                  int32_t* out_grid, hawk_stats* stats) {
    if (!c) return HAWK_EINVAL;
    HAWK_LIVE(c);
    if (c->phase < 1) return fail(c, HAWK_ESTATE, "hawk_generate before hawk_load");
    if (!cond || (c->cfg.use_cfg && !uncond)) return fail(c, HAWK_EINVAL, "null input");
    int rc = check_image_args(c, batch, n_cond, grid_h, grid_w, temperature, top_k, cfg_scale);
    if (rc) return rc;
    if (k < 0 || k > c->kmax || k > grid_w)
        return fail(c, HAWK_EINVAL, "k = %d outside [0, min(k_max = %d, grid_w = %d)]", k, c->kmax, grid_w);
    const int N = grid_h * grid_w;
    if (replay_tokens) {
        for (size_t i = 0; i < (size_t)batch * N; ++i)
            if (replay_tokens[i] < c->cfg.samp_lo || replay_tokens[i] >= c->cfg.samp_lo + c->Vs)
                return fail(c, HAWK_EINVAL, "replayed token outside the sampled slice");
        rc = upload(c, c->off.replay, replay_tokens, (size_t)batch * N * 4);
        if (rc) return rc;
    }
    UniformSrc us;
    memset(&us, 0, sizeof us);
    us.use_gen = 1;
    us.seed = seed;
    us.step = wsp<int32_t>(c, c->off.step);
    HIP_TRY(c, hipEventRecord(c->ev[0], c->stream));
    rc = enqueue_prefill(c, cond, uncond, batch, n_cond, grid_h, grid_w, temperature, top_k, cfg_scale, us);
    if (rc) return rc;
    HIP_TRY(c, hipEventRecord(c->ev[1], c->stream));
    // Every iteration commits at least one token per unfinished prompt, so N-1 iterations
    // always suffice; the committed counts are polled every few iterations to stop early.
    int32_t* nb = static_cast<int32_t*>(c->pinned);
    const DraftMode dm = {replay_tokens ? 2 : 0, replay_tokens ? 1 : 0};
    const int poll = 4;
    bool done = N <= 1;
    for (int it = 0; it < N - 1 && !done; ++it) {
        enqueue_draft(c, k, us, dm);
        enqueue_verify(c, k, us);
        if ((it + 1) % poll == 0 || it == N - 2) {
            HIP_TRY(c, hipGetLastError());
            rc = download(c, nb, c->off.n, (size_t)batch * 4);
            if (rc) return rc;
            done = true;
            for (int b = 0; b < batch; ++b) done = done && nb[b] >= N;
        }
    }
    HIP_TRY(c, hipEventRecord(c->ev[2], c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    c->k_last = k;
    c->phase = 2;
    rc = check_stream(c);
    if (rc) return rc;
    if (out_grid) {
        rc = download(c, out_grid, c->off.grid, (size_t)batch * N * 4);  // rows are N long: N == c->N
        if (rc) return rc;
    }
    if (stats) {
        unsigned long long cnt[4];
        rc = download(c, cnt, c->off.counters, sizeof cnt);
        if (rc) return rc;
        stats->steps = (int64_t)cnt[0];
        stats->accepted = (int64_t)cnt[1];
        stats->tokens = (int64_t)cnt[2];
        stats->iters = (int64_t)cnt[3];
        HIP_TRY(c, hipEventElapsedTime(&stats->ms_prefill, c->ev[0], c->ev[1]));
        HIP_TRY(c, hipEventElapsedTime(&stats->ms_decode, c->ev[1], c->ev[2]));
    }
    return HAWK_OK;
}

int hawk_set_replay(hawk_ctx* c, const int32_t* replay_tokens) {
    if (!c) return HAWK_EINVAL;
    HAWK_LIVE(c);
    if (c->phase < 2) return fail(c, HAWK_ESTATE, "no image in progress");
    if (!replay_tokens) return fail(c, HAWK_EINVAL, "null tokens");
    for (size_t i = 0; i < (size_t)c->B * c->N; ++i)
        if (replay_tokens[i] < c->cfg.samp_lo || replay_tokens[i] >= c->cfg.samp_lo + c->Vs)
            return fail(c, HAWK_EINVAL, "replayed token outside the sampled slice");
    return upload(c, c->off.replay, replay_tokens, (size_t)c->B * c->N * 4);
}

int hawk_run_steps(hawk_ctx* c, int k, int n_steps, uint64_t seed, int replay, float* ms_draft, float* ms_verify,
                   float* ms_kernel) {
    if (!c) return HAWK_EINVAL;
    HAWK_LIVE(c);
    if (c->phase != 2) return fail(c, HAWK_ESTATE, "hawk_run_steps needs a prefilled context with no draft pending");
    if (k < 0 || k > c->kmax || k > c->gw)
        return fail(c, HAWK_EINVAL, "k = %d outside [0, min(k_max = %d, grid_w = %d)]", k, c->kmax, c->gw);
    if (n_steps < 0 || n_steps > 1 << 20) return fail(c, HAWK_EINVAL, "n_steps out of range");
    const bool timed = ms_draft && ms_verify;
    if (timed && (size_t)(4 * n_steps + 1) > c->n_tev) {
        size_t want = (size_t)(4 * n_steps + 1);
        hipEvent_t* ev = static_cast<hipEvent_t*>(realloc(c->tev, want * sizeof(hipEvent_t)));
        if (!ev) return fail(c, HAWK_ENOMEM, "out of host memory");
        c->tev = ev;
        for (; c->n_tev < want; ++c->n_tev) HIP_TRY(c, hipEventCreate(&c->tev[c->n_tev]));
    }
    UniformSrc us;
    memset(&us, 0, sizeof us);
    us.use_gen = 1;
    us.seed = seed;
    us.step = wsp<int32_t>(c, c->off.step);
    const DraftMode dm = {replay ? 2 : 0, replay ? 1 : 0};
    if (timed) HIP_TRY(c, hipEventRecord(c->tev[0], c->stream));
    for (int it = 0; it < n_steps; ++it) {
        enqueue_draft(c, k, us, dm);
        if (timed) {
            HIP_TRY(c, hipEventRecord(c->tev[2 * it + 1], c->stream));
            c->kev_a = c->tev[2 * n_steps + 1 + 2 * it];
            c->kev_b = c->tev[2 * n_steps + 2 + 2 * it];
        }
        enqueue_verify(c, k, us);
        c->kev_a = c->kev_b = nullptr;
        if (timed) HIP_TRY(c, hipEventRecord(c->tev[2 * it + 2], c->stream));
    }
    HIP_TRY(c, hipGetLastError());
    c->k_last = k;
    if (timed) {
        HIP_TRY(c, hipStreamSynchronize(c->stream));
        double md = 0.0, mv = 0.0;
        for (int it = 0; it < n_steps; ++it) {
            float a = 0.f, b = 0.f;
            HIP_TRY(c, hipEventElapsedTime(&a, c->tev[2 * it], c->tev[2 * it + 1]));
            HIP_TRY(c, hipEventElapsedTime(&b, c->tev[2 * it + 1], c->tev[2 * it + 2]));
            md += a;
            mv += b;
        }
        *ms_draft = (float)md;
        *ms_verify = (float)mv;
        if (ms_kernel) {  // the persistent target-pass kernel alone (0 when the generic kernels ran)
            double mk = 0.0;
            if (c->last_path == 1)
                for (int it = 0; it < n_steps; ++it) {
                    float a = 0.f;
                    HIP_TRY(c, hipEventElapsedTime(&a, c->tev[2 * n_steps + 1 + 2 * it], c->tev[2 * n_steps + 2 + 2 * it]));
                    mk += a;
                }
            *ms_kernel = (float)mk;
        }
        return check_stream(c);
    }
    return HAWK_OK;
}

int hawk_get_stats(hawk_ctx* c, hawk_stats* out) {
    if (!c || !out) return HAWK_EINVAL;
    HAWK_LIVE(c);
    if (c->phase < 2) return fail(c, HAWK_ESTATE, "no image in progress");
    unsigned long long cnt[4];
    int rc = download(c, cnt, c->off.counters, sizeof cnt);
    if (rc) return rc;
    memset(out, 0, sizeof *out);
    out->steps = (int64_t)cnt[0];
    out->accepted = (int64_t)cnt[1];
    out->tokens = (int64_t)cnt[2];
    out->iters = (int64_t)cnt[3];
    return check_stream(c);
}

int hawk_get_n(hawk_ctx* c, int32_t* n) {
    if (!c || !n) return HAWK_EINVAL;
    HAWK_LIVE(c);
    if (c->phase < 2) return fail(c, HAWK_ESTATE, "no image in progress");
    return download(c, n, c->off.n, (size_t)c->B * 4);
}

int hawk_get_grid(hawk_ctx* c, int32_t* grid) {
    if (!c || !grid) return HAWK_EINVAL;
    HAWK_LIVE(c);
    if (c->phase < 2) return fail(c, HAWK_ESTATE, "no image in progress");
    return download(c, grid, c->off.grid, (size_t)c->B * c->N * 4);
}

int hawk_get_logits(hawk_ctx* c, float* out, int rows) {
    if (!c || !out) return HAWK_EINVAL;
    HAWK_LIVE(c);
    if (c->phase < 2) return fail(c, HAWK_ESTATE, "no image in progress");
    if (rows < 1 || rows > c->kmax + 1) return fail(c, HAWK_EINVAL, "rows outside [1, k_max + 1]");
    for (int b = 0; b < c->B; ++b) {
        int rc = download(c, out + (size_t)b * rows * c->Vs,
                          c->off.logit_b + (size_t)b * (c->kmax + 1) * c->Vs * 4, (size_t)rows * c->Vs * 4);
        if (rc) return rc;
    }
    return HAWK_OK;
}

int hawk_get_tree_logits(hawk_ctx* c, float* out, int n_nodes) {
    if (!c || !out) return HAWK_EINVAL;
    HAWK_LIVE(c);
    if (c->phase < 2) return fail(c, HAWK_ESTATE, "no image in progress");
    if (n_nodes < 1 || n_nodes > c->kmax + 1) return fail(c, HAWK_EINVAL, "n_nodes outside [1, k_max + 1]");
    if (!c->cfg.use_cfg) return download(c, out, c->off.logit_s, (size_t)c->B * n_nodes * c->Vs * 4);
    // guided rows of all nodes, formed like the rows the walk used
    std::vector<int32_t> all((size_t)c->B * n_nodes);
    for (size_t i = 0; i < all.size(); ++i) all[i] = (int32_t)i;
    int rc = upload(c, c->off.forced, all.data(), all.size() * 4);
    if (rc) return rc;
    launch_gather_rows(c, wsp<float>(c, c->off.logit_s), wsp<int32_t>(c, c->off.forced), wsp<float>(c, c->off.logit_b),
                       c->B * n_nodes, c->Vs, c->B * n_nodes);
    HIP_TRY(c, hipGetLastError());
    return download(c, out, c->off.logit_b, (size_t)c->B * n_nodes * c->Vs * 4);
}

int hawk_get_tree_path(hawk_ctx* c, int32_t* out) {
    if (!c || !out) return HAWK_EINVAL;
    HAWK_LIVE(c);
    if (c->phase < 2) return fail(c, HAWK_ESTATE, "no image in progress");
    return download(c, out, c->off.tree + TreeArea(c).path, (size_t)c->B * kTreeMaxDepth * 4);
}

int hawk_last_hidden(hawk_ctx* c, const void** device_ptr, int* elem_bytes) {
    if (!c || !device_ptr || !elem_bytes) return HAWK_EINVAL;
    HAWK_LIVE(c);
    if (c->phase < 2) return fail(c, HAWK_ESTATE, "no image in progress");
    *device_ptr = c->ws + c->off.x;
    *elem_bytes = (int)c->asz;
    return HAWK_OK;
}

int hawk_get_draft_logits(hawk_ctx* c, float* out, int k) {
    if (!c || !out) return HAWK_EINVAL;
    HAWK_LIVE(c);
    if (c->phase < 2) return fail(c, HAWK_ESTATE, "no image in progress");
    if (k < 1 || k > c->kmax) return fail(c, HAWK_EINVAL, "k outside [1, k_max]");
    for (int b = 0; b < c->B; ++b) {
        int rc = download(c, out + (size_t)b * k * c->Vs, c->off.dlogit_b + (size_t)b * (c->kmax + 1) * c->Vs * 4,
                          (size_t)k * c->Vs * 4);
        if (rc) return rc;
    }
    return HAWK_OK;
}

}  // extern "C"
