// The whole drafting and verification scheme over one image as one library call (Method, overview
// figure: dual-direction heads -> speculation cache -> spatial sampling pool -> one candidate per pool
// member -> candidate tree -> verification), composed from the entry points that implement its parts.
// Host code: the loop, the counter-based uniforms and the bookkeeping of which rows were committed; the
// only kernel here gathers the committed rows' hidden states for the heads.
#include <math.h>
#include <stdio.h>
#include <string.h>

#include <vector>

#include "hawk_internal.h"

namespace hawk {

namespace {

// hidden rows rows[i] of the last pass (elements of 4 or 8 bytes) as fp32 [n_rows][d]
__global__ void gather_hidden_kernel(const void* src, int elem_bytes, const int32_t* rows, int d, float* out) {
    const int r = blockIdx.x, row = rows[r];
    for (int j = threadIdx.x; j < d; j += blockDim.x)
        out[(size_t)r * d + j] = elem_bytes == 8 ? (float)static_cast<const double*>(src)[(size_t)row * d + j]
                                                 : static_cast<const float*>(src)[(size_t)row * d + j];
}

uint64_t mix64(uint64_t z) {   // the splitmix64 finaliser
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}
// The generator hawk_generate documents: u(seed, prompt, step, slot).
float gen_uniform_host(uint64_t seed, uint32_t seq, uint32_t step, uint32_t slot) {
    const uint64_t ctr = ((uint64_t)seq << 44) | ((uint64_t)step << 8) | (uint64_t)(slot & 0xFFu);
    uint64_t z = mix64(seed + 0x9E3779B97F4A7C15ull);
    z = mix64(z + 0x9E3779B97F4A7C15ull * (ctr + 1));
    return (float)(z >> 40) * (1.0f / 16777216.0f);
}

size_t up256(size_t x) { return (x + 255) & ~(size_t)255; }

struct SchemeArea {
    size_t h_rows, q_all, pool, packed, pool_m, pool_delta, cand, u, pos, tgt, sel, heads_ws, cache, total;
    size_t heads_ws_bytes;
    SchemeArea(int d, int Vs, int IW, int HD, int VSD) {
        const int rows = HD + 1, n_heads = HD + VSD, m_max = VSD + 1;
        size_t at = 0;
        auto take = [&](size_t n) { size_t a = at; at = up256(at + n); return a; };
        h_rows = take((size_t)rows * d * 4);
        q_all = take((size_t)rows * n_heads * Vs * 4);
        pool = take((size_t)HD * m_max * Vs * 4);
        packed = take((size_t)HD * m_max * Vs * 4);
        pool_m = take((size_t)HD * 4);
        pool_delta = take((size_t)HD * m_max * 4);
        cand = take((size_t)HD * m_max * 4);
        u = take((size_t)HD * m_max * 4);
        pos = take((size_t)rows * 4);
        tgt = take((size_t)HD * 4);
        sel = take((size_t)rows * 4);
        heads_ws_bytes = hawk_spatial_heads_workspace_bytes(rows, n_heads, d);
        heads_ws = take(heads_ws_bytes);
        cache = take(hawk_spec_cache_bytes(IW, VSD > 0 ? VSD : 1, Vs));
        total = at;
    }
};

int tree_rows(int HD, int VSD) {   // rows of the widest tree: 1 + m + m^2 + ... with m = VSD + 1 candidates per depth
    long n = 1, w = 1;
    for (int j = 0; j < HD; ++j) {
        w *= VSD + 1;
        n += w;
        if (n > 4096) return 4096;
    }
    return (int)n;
}

}  // namespace

}  // namespace hawk

using namespace hawk;

// the first failing step, for hawk_last_error (the context-free entry points leave no message of their own)
static int failed_at(hawk_ctx* c, int rc, const char* what) {
    if (c->err[0] == 0 || strstr(what, "hawk_spatial") || strstr(what, "hawk_spec") || strstr(what, "hawk_sample") ||
        strstr(what, "argument") || strstr(what, "copy") || strstr(what, "workspace"))
        snprintf(c->err, sizeof c->err, "hawk_generate_spatial: %s (code %d)", what, rc);
    return rc;
}

extern "C" {

size_t hawk_generate_spatial_workspace_bytes(const hawk_config* cfg, int grid_w, int HD, int VSD) {
    if (!cfg || HD < 1 || HD > kTreeMaxDepth || VSD < 0 || VSD > 7 || grid_w < 1) return 0;
    const int Vs = cfg->samp_n > 0 ? cfg->samp_n : cfg->vocab;
    return SchemeArea(cfg->d_model, Vs, grid_w, HD, VSD).total;
}

int hawk_generate_spatial(hawk_ctx* c, const float* cond, int n_cond, int grid_h, int grid_w, float temperature, int top_k,
                          const void* W_heads, const void* W_out, int HD, int VSD, uint64_t seed, void* workspace,
                          size_t workspace_bytes, int32_t* out_grid, int64_t* out_stats) {
    if (!c || !cond || !W_heads || !W_out || !workspace || !out_grid) return HAWK_EINVAL;
    if (c->cfg.use_cfg) return failed_at(c, HAWK_EINVAL, "argument: the context was created with guidance");
    if (HD < 1 || HD > kTreeMaxDepth || VSD < 0 || VSD > 7) return failed_at(c, HAWK_EINVAL, "argument: HD outside 1..8 or VSD outside 0..7");
    if (((uintptr_t)workspace & 255) != 0) return failed_at(c, HAWK_EINVAL, "argument: workspace not 256-byte aligned");
    const int d = c->d, Vs = c->Vs, IW = grid_w, IH = grid_h, N = grid_w * grid_h;
    const int n_heads = HD + VSD, m_max = VSD + 1, max_nodes = tree_rows(HD, VSD);
    if (max_nodes > c->kmax + 1 || max_nodes > kTreeMaxNodes)
        return failed_at(c, HAWK_EINVAL, "argument: the widest tree has more rows than the context's k_max + 1 (or than 64)");
    const SchemeArea A(d, Vs, IW, HD, VSD);
    if (workspace_bytes < A.total) return failed_at(c, HAWK_ENOMEM, "workspace too small");
    uint8_t* ws = static_cast<uint8_t*>(workspace);
    hipStream_t st = c->stream;
    float* h_rows = reinterpret_cast<float*>(ws + A.h_rows);
    float* q_all = reinterpret_cast<float*>(ws + A.q_all);
    float* pool = reinterpret_cast<float*>(ws + A.pool);
    float* packed = reinterpret_cast<float*>(ws + A.packed);
    int32_t* pool_m = reinterpret_cast<int32_t*>(ws + A.pool_m);
    int32_t* pool_delta = reinterpret_cast<int32_t*>(ws + A.pool_delta);
    int32_t* cand_dev = reinterpret_cast<int32_t*>(ws + A.cand);
    float* u_dev = reinterpret_cast<float*>(ws + A.u);
    int32_t* pos_dev = reinterpret_cast<int32_t*>(ws + A.pos);
    int32_t* tgt_dev = reinterpret_cast<int32_t*>(ws + A.tgt);
    int32_t* sel_dev = reinterpret_cast<int32_t*>(ws + A.sel);
    void* cache = ws + A.cache;

    // Small host <-> device traffic goes through one page-locked block of its own (the context's is used by
    // the tree step): uploads are asynchronous, each from a slot of its own that is rewritten only after the
    // pass's read-back has synchronised the stream.
    struct Pinned {
        void* p = nullptr;
        ~Pinned() { if (p) (void)hipHostFree(p); }
    } pin;
    if (hipHostMalloc(&pin.p, 4096, hipHostMallocDefault) != hipSuccess) return failed_at(c, HAWK_EDEVICE, "copy or bookkeeping failed");
    size_t pin_at = 0;
    auto up = [&](void* dst, const void* src, size_t bytes) {
        if (pin_at + bytes > 2048) return false;
        void* slot = static_cast<char*>(pin.p) + pin_at;
        pin_at += (bytes + 15) & ~(size_t)15;
        memcpy(slot, src, bytes);
        return hipMemcpyAsync(dst, slot, bytes, hipMemcpyHostToDevice, st) == hipSuccess;
    };
    auto down2 = [&](void* dst_a, const void* src_a, size_t bytes_a, void* dst_b, const void* src_b, size_t bytes_b) {
        char* a = static_cast<char*>(pin.p) + 2048;
        char* b = a + 1024;
        if (bytes_a > 1024 || bytes_b > 1024) return false;
        if (hipMemcpyAsync(a, src_a, bytes_a, hipMemcpyDeviceToHost, st) != hipSuccess ||
            hipMemcpyAsync(b, src_b, bytes_b, hipMemcpyDeviceToHost, st) != hipSuccess || hipStreamSynchronize(st) != hipSuccess)
            return false;
        memcpy(dst_a, a, bytes_a);
        memcpy(dst_b, b, bytes_b);
        pin_at = 0;   // everything uploaded so far has been consumed
        return true;
    };

    const float u0 = gen_uniform_host(seed, 0, 0, kSlotFinal);
    int rc = hawk_prefill(c, cond, nullptr, 1, n_cond, grid_h, grid_w, temperature, top_k, 1.0f, &u0);
    if (rc) return rc;
    if (VSD > 0 && (rc = hawk_spec_cache_reset(cache, IW, VSD, Vs, st)) != 0) return failed_at(c, rc, "hawk_spec_cache_reset");

    int64_t passes = 0, accepted = 0, tail_steps = 0;
    int n = 1, n_rows = 1;
    int32_t sel[kTreeMaxDepth + 1] = {n_cond - 1};   // rows of the last pass that were committed: the prefill's last condition row
    int32_t positions[kTreeMaxDepth + 1] = {0};      // the positions their hidden states predicted
    uint32_t step = 0;
    while (n + max_nodes <= N) {
        ++step;
        // heads on the committed rows; their vertical predictions go to the cache
        const void* hid = nullptr;
        int eb = 0;
        if ((rc = hawk_last_hidden(c, &hid, &eb)) != 0) return rc;
        if (!up(sel_dev, sel, (size_t)n_rows * 4) || !up(pos_dev, positions, (size_t)n_rows * 4)) return failed_at(c, HAWK_EDEVICE, "copy or bookkeeping failed");
        gather_hidden_kernel<<<n_rows, 256, 0, st>>>(hid, eb, sel_dev, d, h_rows);
        if ((rc = hawk_spatial_heads(h_rows, W_heads, W_out, n_rows, n_heads, d, Vs, q_all, nullptr, ws + A.heads_ws,
                                     A.heads_ws_bytes, st)) != 0)
            return failed_at(c, rc, "hawk_spatial_heads");
        if (VSD > 0 && (rc = hawk_spec_cache_push(cache, IW, IH, VSD, Vs, pos_dev, q_all + (size_t)HD * Vs, (size_t)n_heads * Vs,
                                                  n_rows, st)) != 0)
            return failed_at(c, rc, "hawk_spec_cache_push");
        // pools at the HD positions ahead: cached vertical predictions, then the last row's horizontal head
        int32_t targets[kTreeMaxDepth];
        for (int j = 0; j < HD; ++j) targets[j] = n + j;
        if (!up(tgt_dev, targets, (size_t)HD * 4)) return failed_at(c, HAWK_EDEVICE, "copy or bookkeeping failed");
        const float* q_h = q_all + (size_t)(n_rows - 1) * n_heads * Vs;
        if (VSD > 0) {
            if ((rc = hawk_spec_pool(cache, IW, IH, VSD, Vs, tgt_dev, q_h, (size_t)Vs, HD, pool, pool_m, pool_delta, st)) != 0)
                return failed_at(c, rc, "hawk_spec_pool");
        } else {   // no vertical heads: every pool is the horizontal proposal alone
            int32_t ones[kTreeMaxDepth], zeros[kTreeMaxDepth];
            for (int j = 0; j < HD; ++j) { ones[j] = 1; zeros[j] = 0; }
            if (hipMemcpyAsync(pool, q_h, (size_t)HD * Vs * 4, hipMemcpyDeviceToDevice, st) != hipSuccess) return failed_at(c, HAWK_EDEVICE, "copy or bookkeeping failed");
            if (!up(pool_m, ones, (size_t)HD * 4) || !up(pool_delta, zeros, (size_t)HD * 4)) return failed_at(c, HAWK_EDEVICE, "copy or bookkeeping failed");
        }
        // one candidate per pool member
        float u_cand[kTreeMaxDepth * 8];
        for (int j = 0; j < HD; ++j)
            for (int i = 0; i < m_max; ++i) u_cand[j * m_max + i] = gen_uniform_host(seed, 0, step, kSlotDraft + j * 8 + i);
        if (!up(u_dev, u_cand, (size_t)HD * m_max * 4)) return failed_at(c, HAWK_EDEVICE, "copy or bookkeeping failed");
        if ((rc = hawk_sample_rows(pool, pool_delta, u_dev, HD * m_max, Vs, temperature, top_k, cand_dev, st)) != 0)
            return failed_at(c, rc, "hawk_sample_rows");
        int32_t m_host[kTreeMaxDepth], cand_all[kTreeMaxDepth * 8];
        if (!down2(m_host, pool_m, (size_t)HD * 4, cand_all, cand_dev, (size_t)HD * m_max * 4)) return failed_at(c, HAWK_EDEVICE, "copy or bookkeeping failed");
        int mm = 1;
        for (int j = 0; j < HD; ++j) {
            if (m_host[j] < 1 || m_host[j] > m_max) return failed_at(c, HAWK_EDEVICE, "copy or bookkeeping failed");   // cannot happen: the horizontal member always exists
            mm = m_host[j] > mm ? m_host[j] : mm;
        }
        int32_t cand_h[kTreeMaxDepth * 8];
        float u_acc[kTreeMaxDepth * 8], u_fin[kTreeMaxDepth + 1];
        for (int j = 0; j < HD; ++j)
            for (int i = 0; i < mm; ++i) {
                const int cv = cand_all[j * m_max + i];
                cand_h[j * mm + i] = (i < m_host[j] && cv >= 0) ? cv : 0;
                u_acc[j * mm + i] = gen_uniform_host(seed, 0, step, kSlotAcc + j * 8 + i);
            }
        for (int j = 0; j <= HD; ++j) u_fin[j] = gen_uniform_host(seed, 0, step, kSlotFinal + j);
        const float* q_tree = pool;
        if (mm != m_max) {   // the tree step takes [depth][prompt][widest list][V_s] without gaps
            if (hipMemcpy2DAsync(packed, (size_t)mm * Vs * 4, pool, (size_t)m_max * Vs * 4, (size_t)mm * Vs * 4, HD,
                                 hipMemcpyDeviceToDevice, st) != hipSuccess)
                return failed_at(c, HAWK_EDEVICE, "copy or bookkeeping failed");
            q_tree = packed;
        }
        int32_t na = 0, toks[kTreeMaxDepth + 1], path[kTreeMaxDepth];
        if ((rc = hawk_verify_tree(c, HD, m_host, cand_h, q_tree, u_acc, u_fin, &na, toks)) != 0) return rc;
        if ((rc = hawk_get_tree_path(c, path)) != 0) return rc;
        if (na < 0 || na > HD) return failed_at(c, HAWK_EDEVICE, "copy or bookkeeping failed");
        // committed rows of this pass: the root and the accepted candidates' nodes
        sel[0] = 0;
        for (int i = 0; i < na; ++i) sel[i + 1] = path[i];
        n_rows = na + 1;
        for (int i = 0; i <= na; ++i) positions[i] = n + i;
        n += na + 1;
        passes += 1;
        accepted += na;
    }
    while (n < N) {   // the last positions, where the widest tree no longer fits: ordinary steps with one draft token
        ++step;
        const float ud = gen_uniform_host(seed, 0, step, kSlotDraft), ua = gen_uniform_host(seed, 0, step, kSlotAcc),
                    uf = gen_uniform_host(seed, 0, step, kSlotFinal);
        int32_t na = 0;
        if ((rc = hawk_draft(c, 1, &ud, nullptr)) != 0) return rc;
        if ((rc = hawk_verify(c, 1, &ua, &uf, &na, nullptr)) != 0) return rc;
        if (na < 0) break;
        n += na + 1;
        tail_steps += 1;
    }
    if ((rc = hawk_get_grid(c, out_grid)) != 0) return rc;
    if (out_stats) {
        out_stats[0] = passes; out_stats[1] = accepted; out_stats[2] = tail_steps; out_stats[3] = N;
    }
    return HAWK_OK;
}

}  // extern "C"
