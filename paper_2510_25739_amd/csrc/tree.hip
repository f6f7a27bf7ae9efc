// Tree verification (Method, "Spatial Sampling Pool": the candidate tree; "Sampling and
// Verification": the walk): the small kernels around the target pass over the tree's rows - picking
// the target row of the node the walk stands on, moving the accepted path's cache entries into
// place, committing the emitted tokens.  The pass itself runs on the one-kernel-per-operation path
// with tree rows (see RowMap), the per-depth decision is hawk_multi_verify's.
#include "hawk_internal.h"

namespace hawk {

namespace {

// dst[r][0..n) = src[index[r]][0..n); rows with a negative index are left alone.  With guidance
// (uncond_shift > 0: the unconditional stream's row lies that many rows further on) the row is the
// guided combination lu + scale (lc - lu), formed as in the sampling kernels.
__global__ __launch_bounds__(256) void gather_rows_kernel(const float* src, const int32_t* index, float* dst, int n,
                                                          int uncond_shift, float scale) {
    const int r = blockIdx.x, i = index[r];
    if (i < 0) return;
    const float* s = src + (size_t)i * n;
    const float* su = src + (size_t)(i + uncond_shift) * n;
    float* d = dst + (size_t)r * n;
    for (int e = blockIdx.y * 256 + threadIdx.x; e < n; e += 256 * gridDim.y)   // a row is spread over gridDim.y workgroups
        d[e] = uncond_shift > 0 ? fmaf(scale, s[e] - su[e], su[e]) : s[e];
}

// The pass wrote node r's keys and values to the entry root + r.  The accepted path's nodes
// path[0] < path[1] < ... (path[j] >= j + 1) belong at root + 1, root + 2, ...: moved in that order,
// so that no entry is overwritten before it has been moved; each thread moves its own elements of
// every entry, so no synchronisation is needed between the moves.  Block (head, sequence, layer);
// cache layout [layer][sequence][head][entry][hd], elements of `words` 16-bit units.
__global__ __launch_bounds__(256) void kv_compact_kernel(uint16_t* Kc, uint16_t* Vc, const int32_t* n, const int32_t* acc,
                                                         const int32_t* path, int B, int Smax, int H, int Tmax,
                                                         int words, int n_cond) {
    const int h = blockIdx.x, s = blockIdx.y, layer = blockIdx.z, b = s % B;
    const int a = acc[b];
    if (a <= 0) return;
    const int root = n_cond + n[b] - 1;
    const size_t base = (((size_t)layer * Smax + s) * H + h) * (size_t)Tmax * words;
    for (int j = 1; j <= a; ++j) {
        const int node = path[b * kTreeMaxDepth + j - 1];
        if (node == j) continue;
        const size_t src = base + (size_t)(root + node) * words, dst = base + (size_t)(root + j) * words;
        for (int e = threadIdx.x; e < words; e += 256) {
            Kc[dst + e] = Kc[src + e];
            Vc[dst + e] = Vc[src + e];
        }
    }
}

// One round of the walk for every prompt (thread b), after the verification of depth j + 1 (or, for
// j = depth, after the draw of the extra token): the token of the round is recorded; an accepted
// candidate moves the prompt to that child - children of a node lie next to each other in candidate
// order, depth by depth - and gives it the next depth's candidates; otherwise its walk is over.
// meta: depth, nodes, widest list, then first node of every depth (from word 3) and the number of
// candidates per depth (from word 16).  state: [word][B] with words cur (row of the node the prompt
// stands on), rows (candidates in the coming round), idx, tok (the verification's results),
// walking, acc.
__global__ void tree_advance_kernel(const int32_t* meta, int32_t* state, int32_t* path, int32_t* toks, int j, int B,
                                    int samp_lo) {
    const int b = threadIdx.x;
    if (b >= B) return;
    int32_t *cur = state, *rows = state + B, *idx = state + 2 * B, *tok = state + 3 * B, *walking = state + 4 * B,
            *acc = state + 5 * B;
    if (!walking[b]) return;
    const int depth = meta[0], n_nodes = meta[1];
    const int32_t *first = meta + 3, *width = meta + 16;
    const int a = acc[b];
    toks[b * (kTreeMaxDepth + 1) + a] = samp_lo + tok[b];
    if (j < depth && idx[b] < width[j]) {
        const int here = a > 0 ? path[b * kTreeMaxDepth + a - 1] : 0;
        const int node = first[j + 1] + (here - first[j]) * width[j] + idx[b];
        path[b * kTreeMaxDepth + a] = node;
        acc[b] = a + 1;
        cur[b] = b * n_nodes + node;
        rows[b] = j + 1 < depth ? width[j + 1] : 0;
    } else {
        walking[b] = 0;
        rows[b] = 0;
    }
}

// Prompt b: tokens toks[0..a] into the grid, n += a + 1, the hidden state of the last accepted node
// (the root if none) kept for the next draft, counters as in the chain's commit.
__global__ __launch_bounds__(256) void tree_commit_kernel(const int32_t* acc, const int32_t* path, const int32_t* toks,
                                                          int32_t* grid, int32_t* n, const uint32_t* hid,
                                                          uint32_t* hprev, int hid_words, int n_nodes, int B, int N,
                                                          int n_streams, unsigned long long* counters) {
    const int b = blockIdx.x, a = acc[b];
    if (a < 0) return;
    const int last = a > 0 ? path[b * kTreeMaxDepth + a - 1] : 0;
    for (int s = b; s < n_streams; s += B) {
        const uint32_t* src = hid + ((size_t)s * n_nodes + last) * hid_words;
        uint32_t* dst = hprev + (size_t)s * hid_words;
        for (int i = threadIdx.x; i < hid_words; i += 256) dst[i] = src[i];
    }
    if (threadIdx.x == 0) {
        const int nb = n[b];
        for (int i = 0; i <= a; ++i) grid[(size_t)b * N + nb + i] = toks[b * (kTreeMaxDepth + 1) + i];
        n[b] = nb + a + 1;
        atomicAdd(&counters[0], 1ull);
        atomicAdd(&counters[1], (unsigned long long)a);
        atomicAdd(&counters[2], (unsigned long long)(a + 1));
    }
}

}  // namespace

void launch_gather_rows(hawk_ctx* c, const float* src, const int32_t* index, float* dst, int rows, int n, int uncond_shift) {
    gather_rows_kernel<<<dim3(rows, 16), 256, 0, c->stream>>>(src, index, dst, n, uncond_shift, c->cfg_scale);
}

void launch_tree_advance(hawk_ctx* c, const int32_t* meta, int32_t* state, int32_t* path, int32_t* toks, int j) {
    tree_advance_kernel<<<1, 64 * ((c->B + 63) / 64), 0, c->stream>>>(meta, state, path, toks, j, c->B, c->cfg.samp_lo);
}

void launch_tree_commit(hawk_ctx* c, const int32_t* acc, const int32_t* path, const int32_t* toks, int n_nodes) {
    kv_compact_kernel<<<dim3(c->H, c->S, c->L), 256, 0, c->stream>>>(
        wsp<uint16_t>(c, c->off.kc), wsp<uint16_t>(c, c->off.vc), wsp<int32_t>(c, c->off.n), acc, path, c->B, c->Smax,
        c->H, c->Tmax, (int)(c->hd * c->ksz / 2), c->C);
    tree_commit_kernel<<<c->B, 256, 0, c->stream>>>(acc, path, toks, wsp<int32_t>(c, c->off.grid), wsp<int32_t>(c, c->off.n),
                                                    wsp<uint32_t>(c, c->off.x), wsp<uint32_t>(c, c->off.hprev),
                                                    (int)(c->d * c->asz / 4), n_nodes, c->B, c->N, c->S,
                                                    wsp<unsigned long long>(c, c->off.counters));
}

}  // namespace hawk
