// Generic (any-shape) kernels of the target decoder and the draft head.
//
// Two arithmetic configurations, selected by the weight dtype of the context:
//   fp32 blobs: fp32 weights, fp64 activations / accumulators / KV cache (exact-parity set);
//   bf16 blobs: bf16 weights, fp16 KV cache (same bytes as bf16, 3 more mantissa bits: the
//               cache's rounding is what dominates the logit error), fp32 activations and
//               accumulators.
// One wave computes one output column of a skinny GEMM for up to RT rows, streaming its
// weight row with 16-byte loads; this is the fallback path and the only path of the
// fp32 configuration.  The weight-streaming fast path lives in stream.hip.
#include "hawk_internal.h"

namespace hawk {

struct CfgF32 {
    using WT = float; using AT = double; using KT = double;
    static constexpr int VE = 4;
};
struct CfgBF16 {
    using WT = uint16_t; using AT = float; using KT = _Float16;
    static constexpr int VE = 8;
};

__device__ __forceinline__ float bf16_to_f32(uint32_t b) { return __uint_as_float(b << 16); }
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {  // round to nearest even
    uint32_t u = __float_as_uint(f);
    return (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
}

__device__ __forceinline__ void load_w(const float* p, double* out) {
    float4 v = *reinterpret_cast<const float4*>(p);
    out[0] = v.x; out[1] = v.y; out[2] = v.z; out[3] = v.w;
}
__device__ __forceinline__ void load_w(const uint16_t* p, float* out) {
    uint4 v = *reinterpret_cast<const uint4*>(p);
    out[0] = bf16_to_f32(v.x & 0xFFFFu); out[1] = bf16_to_f32(v.x >> 16);
    out[2] = bf16_to_f32(v.y & 0xFFFFu); out[3] = bf16_to_f32(v.y >> 16);
    out[4] = bf16_to_f32(v.z & 0xFFFFu); out[5] = bf16_to_f32(v.z >> 16);
    out[6] = bf16_to_f32(v.w & 0xFFFFu); out[7] = bf16_to_f32(v.w >> 16);
}
__device__ __forceinline__ double w1(const float* p, size_t i) { return (double)p[i]; }
__device__ __forceinline__ float w1(const uint16_t* p, size_t i) { return bf16_to_f32(p[i]); }
__device__ __forceinline__ double kload(const double* p, size_t i) { return p[i]; }
__device__ __forceinline__ float kload(const _Float16* p, size_t i) { return (float)p[i]; }
__device__ __forceinline__ void kstore(double* p, size_t i, double v) { p[i] = v; }
__device__ __forceinline__ void kstore(_Float16* p, size_t i, float v) { p[i] = (_Float16)v; }

template <typename T> __device__ __forceinline__ T wave_sum(T v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
template <typename T> __device__ __forceinline__ T wave_max(T v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) { T t = __shfl_xor(v, o, 64); v = t > v ? t : v; }
    return v;
}
// Sum over a 256-thread block; every thread gets the result. red: >= 4 entries of LDS.
template <typename T> __device__ __forceinline__ T block_sum256(T v, T* red) {
    v = wave_sum(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    return red[0] + red[1] + red[2] + red[3];
}
template <typename T> __device__ __forceinline__ T block_max256(T v, T* red) {
    v = wave_max(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    T a = red[0] > red[1] ? red[0] : red[1], b = red[2] > red[3] ? red[2] : red[3];
    return a > b ? a : b;
}

// Row R of a pass -> sequence, row within the sequence, prompt, absolute position.
// pos: position (rotary angle); slot: index of the row's entry in the cache (= pos except for tree rows).
struct RowInfo { int s, r, b, pos, slot; bool valid; };
__device__ __forceinline__ RowInfo row_info(const RowMap& m, int R) {
    RowInfo o;
    o.s = R / m.rows_per_seq;
    o.r = R - o.s * m.rows_per_seq;
    o.b = o.s % m.batch;
    if (m.mode == 0) {
        o.pos = o.r;
        o.valid = true;
    } else {
        int ke = m.k_eff[o.b];
        o.valid = o.r <= ke;
        o.pos = o.valid ? m.n_cond + m.n[o.b] - 1 + (m.mode == 2 ? m.tree_depth[o.r] : o.r) : 0;
    }
    o.slot = (m.mode == 2 && o.valid) ? m.n_cond + m.n[o.b] - 1 + o.r : o.pos;
    return o;
}

// ------------------------------------------------------------------ rows in

// X[R] = E[token of row R]: row 0 of a sequence is the last committed token, row r > 0
// is draft r-1.
template <class Cfg>
__global__ void embed_rows_kernel(typename Cfg::AT* X, const typename Cfg::WT* E, RowMap map,
                                  const int32_t* grid, const int32_t* draft, int N, int kstride, int d) {
    RowInfo ri = row_info(map, blockIdx.x);
    int tok = 0;
    if (ri.valid) tok = ri.r == 0 ? grid[(size_t)ri.b * N + map.n[ri.b] - 1] : draft[ri.b * kstride + ri.r - 1];
    if (tok < 0) tok = 0;
    for (int i = threadIdx.x; i < d; i += blockDim.x)
        X[(size_t)blockIdx.x * d + i] = w1(E, (size_t)tok * d + i);
}

template <class Cfg>
__global__ void cond_rows_kernel(typename Cfg::AT* X, const float* cond, size_t total) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < total) X[i] = (typename Cfg::AT)cond[i];
}

template <class Cfg>
__global__ __launch_bounds__(256) void rmsnorm_kernel(const typename Cfg::AT* X, const typename Cfg::WT* g,
                                                      typename Cfg::AT* out, int d, size_t in_stride,
                                                      float eps, uint16_t* hi, uint16_t* lo) {
    using AT = typename Cfg::AT;
    __shared__ AT red[4];
    const AT* x = X + (size_t)blockIdx.x * in_stride;
    AT ss = 0;
    for (int i = threadIdx.x; i < d; i += 256) ss += x[i] * x[i];
    ss = block_sum256(ss, red);
    AT r = (AT)1 / sqrt(ss / (AT)d + (AT)eps);
    for (int i = threadIdx.x; i < d; i += 256) {
        const AT v = x[i] * r * w1(g, i);
        out[(size_t)blockIdx.x * d + i] = v;
        if (hi) {   // bf16 planes of the same row for the GEMM that follows
            unsigned h, l;
            bf16_split((float)v, h, l);
            hi[(size_t)blockIdx.x * d + i] = (uint16_t)h;
            lo[(size_t)blockIdx.x * d + i] = (uint16_t)l;
        }
    }
}

// The same for fp32 activations and bf16 gains with the row held in registers (V float4 per
// thread: d <= 1024 V, d % 4 == 0, rows 16-byte aligned): one pass over the row instead of two
// loops of dependent scalar loads.
template <int V>
__global__ __launch_bounds__(256) void rmsnorm_rows_kernel(const float* X, const uint16_t* g, float* out, int d,
                                                           size_t in_stride, float eps, uint16_t* hi, uint16_t* lo) {
    __shared__ float red[4];
    const float4* x = reinterpret_cast<const float4*>(X + (size_t)blockIdx.x * in_stride);
    const int n4 = d / 4;
    float4 v[V];
    uint2 gw[V];
    float ss = 0.f;
#pragma unroll
    for (int i = 0; i < V; ++i) {
        const int q = threadIdx.x + i * 256;
        v[i] = q < n4 ? x[q] : make_float4(0.f, 0.f, 0.f, 0.f);
        gw[i] = q < n4 ? reinterpret_cast<const uint2*>(g)[q] : make_uint2(0u, 0u);
    }
#pragma unroll
    for (int i = 0; i < V; ++i) ss += v[i].x * v[i].x + v[i].y * v[i].y + v[i].z * v[i].z + v[i].w * v[i].w;
    ss = block_sum256(ss, red);
    const float r = 1.0f / sqrtf(ss / (float)d + eps);
#pragma unroll
    for (int i = 0; i < V; ++i) {
        const int q = threadIdx.x + i * 256;
        if (q < n4) {
            float4 o;
            o.x = v[i].x * r * __uint_as_float(gw[i].x << 16);
            o.y = v[i].y * r * __uint_as_float(gw[i].x & 0xFFFF0000u);
            o.z = v[i].z * r * __uint_as_float(gw[i].y << 16);
            o.w = v[i].w * r * __uint_as_float(gw[i].y & 0xFFFF0000u);
            reinterpret_cast<float4*>(out + (size_t)blockIdx.x * d)[q] = o;
            if (hi) {   // bf16 planes of the same row for the GEMM that follows
                unsigned h0, h1, h2, h3, l0, l1, l2, l3;
                bf16_split(o.x, h0, l0);
                bf16_split(o.y, h1, l1);
                bf16_split(o.z, h2, l2);
                bf16_split(o.w, h3, l3);
                reinterpret_cast<uint2*>(hi + (size_t)blockIdx.x * d)[q] = make_uint2(h0 | (h1 << 16), h2 | (h3 << 16));
                reinterpret_cast<uint2*>(lo + (size_t)blockIdx.x * d)[q] = make_uint2(l0 | (l1 << 16), l2 | (l3 << 16));
            }
        }
    }
}

// ------------------------------------------------------------------ skinny GEMM

template <class Cfg, int RT, typename OT>
__global__ __launch_bounds__(256) void gemm_rows_kernel(const typename Cfg::AT* A, int lda,
                                                        const typename Cfg::WT* W, int N, int K,
                                                        OT* Y, int ldy, int M, int accumulate) {
    using AT = typename Cfg::AT;
    constexpr int VE = Cfg::VE;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int n = blockIdx.x * 4 + wave;
    if (n >= N) return;
    const int r0 = blockIdx.y * RT;
    AT acc[RT];
#pragma unroll
    for (int r = 0; r < RT; ++r) acc[r] = 0;
    const typename Cfg::WT* wrow = W + (size_t)n * K;
    for (int c = lane * VE; c < K; c += 64 * VE) {
        AT w[VE];
        load_w(wrow + c, w);
#pragma unroll
        for (int r = 0; r < RT; ++r) {
            if (r0 + r < M) {
                const AT* a = A + (size_t)(r0 + r) * lda + c;
#pragma unroll
                for (int e = 0; e < VE; ++e) acc[r] += w[e] * a[e];
            }
        }
    }
#pragma unroll
    for (int r = 0; r < RT; ++r) acc[r] = wave_sum(acc[r]);
    if (lane == 0) {
#pragma unroll
        for (int r = 0; r < RT; ++r)
            if (r0 + r < M) {
                OT* y = Y + (size_t)(r0 + r) * ldy + n;
                *y = (OT)((accumulate ? (AT)*y : (AT)0) + acc[r]);
            }
    }
}

// ------------------------------------------------------------------ rotary + cache append

// In place on QKV[R] = [q | k | v]: rotates q and k (pair (2j, 2j+1) of each head by
// pos * inv_freq[j]) and writes k, v to the cache at (sequence, pos).
template <class Cfg>
__global__ void rope_append_kernel(typename Cfg::AT* QKV, typename Cfg::KT* Kc, typename Cfg::KT* Vc,
                                   RowMap map, const double* inv_freq, int layer, int d, int hd,
                                   int Smax, int Tmax) {
    using AT = typename Cfg::AT;
    RowInfo ri = row_info(map, blockIdx.x);
    if (!ri.valid) return;
    AT* q = QKV + (size_t)blockIdx.x * 3 * d;
    AT* k = q + d;
    AT* v = k + d;
    // cache layout [layer][sequence][head][position][hd]: one head's entries are contiguous
    const int H = d / hd;
    auto at = [&](int e) {   // element e of the row (feature index within d)
        const int h = e / hd;
        return ((((size_t)layer * Smax + ri.s) * H + h) * Tmax + ri.slot) * hd + (e - h * hd);
    };
    // the angles depend on the position and the pair index within a head only: one sincos per pair
    // index and row, shared by all heads through LDS (hd <= 512)
    __shared__ double tab_c[256], tab_s[256];
    for (int j = threadIdx.x; j < hd / 2; j += blockDim.x) sincos((double)ri.pos * inv_freq[j], &tab_s[j], &tab_c[j]);
    __syncthreads();
    constexpr int U = 4;   // pairs per thread in flight
    for (int p0 = threadIdx.x; p0 < d / 2; p0 += U * blockDim.x) {
        AT qa[U], qb[U], ka[U], kb[U], va[U], vb[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int p = p0 + u * blockDim.x;
            if (p < d / 2) {
                qa[u] = q[2 * p]; qb[u] = q[2 * p + 1];
                ka[u] = k[2 * p]; kb[u] = k[2 * p + 1];
                va[u] = v[2 * p]; vb[u] = v[2 * p + 1];
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int p = p0 + u * blockDim.x;
            if (p < d / 2) {
                const int j = p % (hd / 2);
                const AT c = (AT)tab_c[j], sn = (AT)tab_s[j];
                q[2 * p] = qa[u] * c - qb[u] * sn;
                q[2 * p + 1] = qa[u] * sn + qb[u] * c;
                kstore(Kc, at(2 * p), ka[u] * c - kb[u] * sn);
                kstore(Kc, at(2 * p + 1), ka[u] * sn + kb[u] * c);
                kstore(Vc, at(2 * p), va[u]);
                kstore(Vc, at(2 * p + 1), vb[u]);
            }
        }
    }
}

// ------------------------------------------------------------------ attention

// One workgroup per (head, row): the row attends cache entries 0..pos of its sequence
// (its own entry included), i.e. causal inside the block of new rows.  Tree rows: entries up to
// the root's, then of the new entries only the row's ancestors and its own.
template <class Cfg>
__global__ __launch_bounds__(256) void attention_kernel(const typename Cfg::AT* QKV, const typename Cfg::KT* Kc,
                                                        const typename Cfg::KT* Vc, typename Cfg::AT* O,
                                                        RowMap map, int layer, int d, int hd, int Smax, int Tmax,
                                                        uint16_t* hi, uint16_t* lo) {
    using AT = typename Cfg::AT;
    extern __shared__ double smem_raw[];
    AT* sc = reinterpret_cast<AT*>(smem_raw);  // [Tmax] scores, then [hd] q, then [256] partials
    AT* sq = sc + Tmax;
    AT* part = sq + hd;
    __shared__ AT red[4];
    const int R = blockIdx.y, h = blockIdx.x, tid = threadIdx.x;
    RowInfo ri = row_info(map, R);
    if (!ri.valid) return;
    const size_t base = ((((size_t)layer * Smax + ri.s) * (d / hd) + h) * Tmax) * hd;   // this head's entries, contiguous
    for (int i = tid; i < hd; i += 256) sq[i] = QKV[(size_t)R * 3 * d + (size_t)h * hd + i];
    __syncthreads();
    const AT scale = (AT)1 / sqrt((AT)hd);
    const int root = ri.slot - ri.r;   // tree rows: entry of node 0
    const unsigned long long anc = map.mode == 2 ? (map.tree_anc[ri.r] | (1ull << ri.r)) : ~0ull;
    AT mx = -INFINITY;
    for (int t = tid; t <= ri.slot; t += 256) {
        AT s = 0;
        for (int i = 0; i < hd; ++i) s += sq[i] * kload(Kc, base + (size_t)t * hd + i);
        s *= scale;
        if (map.mode == 2 && t > root && !((anc >> (t - root)) & 1ull)) s = -INFINITY;   // not on the row's path
        sc[t] = s;
        mx = s > mx ? s : mx;
    }
    mx = block_max256(mx, red);
    AT den = 0;
    for (int t = tid; t <= ri.slot; t += 256) {
        AT e = exp(sc[t] - mx);
        sc[t] = e;
        den += e;
    }
    den = block_sum256(den, red);  // also orders the sc[] writes before the reads below
    const int i = tid % hd, sl = tid / hd, nsl = 256 / hd;
    AT acc = 0;
    for (int t = sl; t <= ri.slot; t += nsl) acc += sc[t] * kload(Vc, base + (size_t)t * hd + i);
    part[tid] = acc;
    __syncthreads();
    if (tid < hd) {
        AT o = 0;
        for (int s2 = 0; s2 < nsl; ++s2) o += part[s2 * hd + tid];
        o /= den;
        O[(size_t)R * d + (size_t)h * hd + tid] = o;
        if (hi) {   // the bf16 planes the projection that follows reads
            unsigned a, b;
            bf16_split((float)o, a, b);
            hi[(size_t)R * d + (size_t)h * hd + tid] = (uint16_t)a;
            lo[(size_t)R * d + (size_t)h * hd + tid] = (uint16_t)b;
        }
    }
}

// v of another lane of the same 16-lane row, chosen by a DPP control: 0xB1 lane ^ 1, 0x4E lane ^ 2
// (quad permutes), 0x141 lane l <-> 7 - l within each 8 lanes, 0x140 l <-> 15 - l within the row.
template <int CTRL> __device__ __forceinline__ float dpp_lane(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}

// Step rows of the bf16 configuration, one workgroup per (sequence, head): the sequence's k+1 new
// rows share one pass over its cached keys and one over its values (a workgroup per row would
// read them k+1 times).  Row r attends entries 0..pos0+r.  RM (4 or 8) >= NR >= rows per sequence:
// storage and lane folds are laid out for RM rows, arithmetic is spent on NR;
// hd = 64 or 128.
template <int RM, int NR>
__global__ __launch_bounds__(256) void attention_rows_kernel(const float* QKV, _Float16* Kc, _Float16* Vc, float* O,
                                                             RowMap map, const double* inv_freq, int layer, int d,
                                                             int hd, int Smax, int Tmax, uint16_t* hi, uint16_t* lo) {
    extern __shared__ double smem_raw[];
    float* sq = reinterpret_cast<float*>(smem_raw);   // [RM][hd] queries
    float* sc = sq + RM * hd;                         // [Tmax][RM] scores, then weights
    float* part = sc + (size_t)Tmax * RM;             // [4 waves][RM][hd] partial outputs
    __shared__ float red[4][RM];
    // sequences along x, heads along y
    const int s = blockIdx.x, h = blockIdx.y, tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int R0 = s * map.rows_per_seq;
    const RowInfo r0 = row_info(map, R0);
    const int nrows = r0.valid ? min(map.k_eff[r0.b] + 1, RM) : 0;
    if (hi)   // rows not in flight: defined planes (their results are never used)
        for (int j = nrows * hd + tid; j < map.rows_per_seq * hd; j += 256) {
            const size_t at = (size_t)(R0 + j / hd) * d + (size_t)h * hd + j % hd;
            hi[at] = 0;
            lo[at] = 0;
        }
    if (!r0.valid) return;
    const int pos0 = r0.pos, last = pos0 + nrows - 1;
    const size_t base = ((((size_t)layer * Smax + s) * (d / hd) + h) * Tmax) * hd;   // this head's entries, contiguous
    // The rows' own rotary step and cache append happen here (QKV holds the raw projections): the
    // workgroup rotates its head's q and k rows (pair (2j, 2j+1) by pos * inv_freq[j], as
    // rope_append_kernel does), keeps q in LDS and writes k, v to the cache, where the passes below
    // read them back like every other entry.
    for (int i = tid; i < RM * (hd / 2); i += 256) {
        const int r = i / (hd / 2), j = i - r * (hd / 2);
        float q0 = 0.f, q1 = 0.f;
        if (r < nrows) {
            double sn, cs;
            sincos((double)(pos0 + r) * inv_freq[j], &sn, &cs);
            const float c = (float)cs, sf = (float)sn;
            const float* row = QKV + (size_t)(R0 + r) * 3 * d + (size_t)h * hd + 2 * j;
            const float qa = row[0], qb = row[1], ka = row[d], kb = row[d + 1];
            q0 = qa * c - qb * sf;
            q1 = qa * sf + qb * c;
            const size_t at = base + (size_t)(pos0 + r) * hd + 2 * j;
            Kc[at] = (_Float16)(ka * c - kb * sf);
            Kc[at + 1] = (_Float16)(ka * sf + kb * c);
            Vc[at] = (_Float16)row[2 * d];
            Vc[at + 1] = (_Float16)row[2 * d + 1];
        }
        sq[r * hd + 2 * j] = q0;
        sq[r * hd + 2 * j + 1] = q1;
    }
    __syncthreads();   // also makes the appended entries visible to the other waves of the workgroup
    const float scale = 1.f / sqrtf((float)hd);
    typedef _Float16 h8 __attribute__((ext_vector_type(8)));
    typedef float f4 __attribute__((ext_vector_type(4)));
    const int cpr = hd / 8;   // 16-byte chunks per cache row of the head
    // Scores on the matrix cores: a tile of 16 cache entries is the A operand (lane (e, g) holds
    // features 32 ks + 8 g .. + 7 of entry t0 + e: 16 bytes straight from the fp16 cache), the
    // query rows - scaled, split into an fp16 hi and lo half so that they keep fp32 accuracy - are
    // the B operand, and the result lane (row, g) holds the scores of entries t0 + 4 g .. + 3.
    // Each wave takes every fourth tile.
    const int r16 = lane & 15, kg = lane >> 4, KS = hd / 32;
    h8 qh[4], ql[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float v = (ks < KS && r16 < RM) ? sq[r16 * hd + ks * 32 + kg * 8 + e] * scale : 0.f;
            const _Float16 h = (_Float16)v;
            qh[ks][e] = h;
            ql[ks][e] = (_Float16)(v - (float)h);
        }
    float mxl = -INFINITY;   // running maximum of row r16 over this lane's entries
    {
        const _Float16* kp = Kc + base + kg * 8;
        const int ntile = last / 16 + 1;
        constexpr int TB = 4;   // tiles requested together: their loads overlap
        for (int ib = wave; ib < ntile; ib += 4 * TB) {
            h8 k8[TB][4];
#pragma unroll
            for (int u = 0; u < TB; ++u) {
                // tiles and entries past the end repeat the last entry (masked below)
                const _Float16* row = kp + (size_t)min((ib + 4 * u) * 16 + r16, last) * hd;
#pragma unroll
                for (int ks = 0; ks < 4; ++ks)
                    if (ks < KS) k8[u][ks] = *reinterpret_cast<const h8*>(row + ks * 32);
            }
#pragma unroll
            for (int u = 0; u < TB; ++u) {
                const int t0 = (ib + 4 * u) * 16;
                f4 acc = (f4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < 4; ++ks)
                    if (ks < KS) {
                        acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(k8[u][ks], qh[ks], acc, 0, 0, 0);
                        acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(k8[u][ks], ql[ks], acc, 0, 0, 0);
                    }
                if (r16 < RM) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int t = t0 + 4 * kg + e;
                        const float v = (t <= last && r16 < nrows && t <= pos0 + r16) ? acc[e] : -INFINITY;
                        if (t <= last) sc[(size_t)t * RM + r16] = v;
                        mxl = fmaxf(mxl, v);
                    }
                }
            }
        }
    }
    // per-row maximum over the workgroup (lanes r, r + 16, r + 32, r + 48 of a wave hold row r)
    mxl = fmaxf(mxl, __shfl_xor(mxl, 16));
    mxl = fmaxf(mxl, __shfl_xor(mxl, 32));
    if (lane < RM) red[wave][lane] = mxl;
    float mx[RM];
    __syncthreads();
    float den[RM];
#pragma unroll
    for (int r = 0; r < RM; ++r) {
        mx[r] = fmaxf(fmaxf(red[0][r], red[1][r]), fmaxf(red[2][r], red[3][r]));
        den[r] = 0.f;
    }
    __syncthreads();
    for (int t = tid; t <= last; t += 256) {
#pragma unroll
        for (int r = 0; r < RM; ++r) {
            const float v = sc[(size_t)t * RM + r];
            const float e = (r < nrows && v != -INFINITY) ? expf(v - mx[r]) : 0.f;
            sc[(size_t)t * RM + r] = e;
            den[r] += e;
        }
    }
#pragma unroll
    for (int r = 0; r < RM; ++r) {
        float v = den[r];
        for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
        if (lane == 0) red[wave][r] = v;
    }
    __syncthreads();   // also orders the sc[] writes before the reads below
#pragma unroll
    for (int r = 0; r < RM; ++r) den[r] = (red[0][r] + red[1][r]) + (red[2][r] + red[3][r]);
    // weighted values: here the lanes that share a feature group sit next to each other (lane =
    // group * slots + slot, a slot takes every nsv-th entry), so that their partial sums fold with
    // DPP moves; a wave still requests whole rows of the head
    const int slots = 64 / cpr, c8v = lane / slots, nsv = 4 * slots, slv = wave * slots + lane % slots;
    float acc[RM][8];
#pragma unroll
    for (int r = 0; r < RM; ++r)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[r][e] = 0.f;
    const _Float16* vp = Vc + base + c8v * 8;
    auto fold = [&](int t, const h8& v) {
        float p[RM];
#pragma unroll
        for (int r = 0; r < RM; r += 4) {
            const float4 q4 = *reinterpret_cast<const float4*>(sc + (size_t)t * RM + r);
            p[r] = q4.x;
            p[r + 1] = q4.y;
            p[r + 2] = q4.z;
            p[r + 3] = q4.w;
        }
#pragma unroll
        for (int r = 0; r < NR; ++r)
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[r][e] += p[r] * (float)v[e];
    };
    int t = slv;
    for (; t + 7 * nsv <= last; t += 8 * nsv) {   // eight entries in flight per lane
        h8 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = *reinterpret_cast<const h8*>(vp + (size_t)(t + u * nsv) * hd);
#pragma unroll
        for (int u = 0; u < 8; ++u) fold(t + u * nsv, v[u]);
    }
    for (; t <= last; t += nsv) fold(t, *reinterpret_cast<const h8*>(vp + (size_t)t * hd));
#pragma unroll
    for (int r = 0; r < RM; ++r)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float v = acc[r][e];
            v += dpp_lane<0xB1>(v);
            v += dpp_lane<0x4E>(v);
            if (slots == 8) v += dpp_lane<0x141>(v);
            acc[r][e] = v;
        }
    if (lane % slots == 0) {
#pragma unroll
        for (int r = 0; r < RM; ++r)
#pragma unroll
            for (int e = 0; e < 8; ++e) part[(wave * RM + r) * hd + c8v * 8 + e] = acc[r][e];
    }
    __syncthreads();
    for (int j = tid; j < nrows * hd; j += 256) {
        const int r = j / hd, c = j - r * hd;
        const float o = (part[r * hd + c] + part[(RM + r) * hd + c]) + (part[(2 * RM + r) * hd + c] + part[(3 * RM + r) * hd + c]);
        const float v = o / den[r];
        const size_t at = (size_t)(R0 + r) * d + (size_t)h * hd + c;
        O[at] = v;
        if (hi) {   // bf16 planes for the Wo GEMM that follows
            unsigned hh, ll;
            bf16_split(v, hh, ll);
            hi[at] = (uint16_t)hh;
            lo[at] = (uint16_t)ll;
        }
    }
}

template <class Cfg>
__global__ void swiglu_kernel(typename Cfg::AT* U, int m, size_t total, uint16_t* hi, uint16_t* lo) {
    using AT = typename Cfg::AT;
    size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    size_t row = idx / m, i = idx - row * m;
    AT a = U[row * 2 * m + i], b = U[row * 2 * m + m + i];
    const AT v = a / ((AT)1 + exp(-a)) * b;
    U[row * 2 * m + i] = v;
    if (hi) {   // bf16 planes [row][m] for the GEMM that follows
        unsigned h, l;
        bf16_split((float)v, h, l);
        hi[idx] = (uint16_t)h;
        lo[idx] = (uint16_t)l;
    }
}

// ------------------------------------------------------------------ draft head input

// DIN[s] = [previous head output (target hidden for the first draft) | E[left] | E[up]]
// for draft i (1-based) of every sequence.
template <class Cfg>
__global__ void draft_input_kernel(typename Cfg::AT* DIN, const typename Cfg::AT* prev,
                                   const typename Cfg::WT* E, const int32_t* n_arr, const int32_t* k_eff,
                                   const int32_t* grid, const int32_t* draft, int i, int B, int N, int IW,
                                   int kstride, int d) {
    using AT = typename Cfg::AT;
    const int s = blockIdx.x, b = s % B;
    AT* out = DIN + (size_t)s * 3 * d;
    if (i > k_eff[b]) {
        for (int c = threadIdx.x; c < 3 * d; c += blockDim.x) out[c] = 0;
        return;
    }
    const int n = n_arr[b], t = n - 1 + i;
    const int left = (i == 1) ? grid[(size_t)b * N + n - 1] : draft[b * kstride + i - 2];
    const int up = (t >= IW) ? grid[(size_t)b * N + t - IW] : -1;
    for (int c = threadIdx.x; c < d; c += blockDim.x) {
        out[c] = prev[(size_t)s * d + c];
        out[d + c] = w1(E, (size_t)left * d + c);
        out[2 * d + c] = up >= 0 ? w1(E, (size_t)up * d + c) : (AT)0;
    }
}

template <class Cfg>
__global__ void keep_hprev_prefill_kernel(typename Cfg::AT* hprev, const typename Cfg::AT* X, int C, int d) {
    const int s = blockIdx.x;
    for (int c = threadIdx.x; c < d; c += blockDim.x)
        hprev[(size_t)s * d + c] = X[((size_t)s * C + C - 1) * d + c];
}

// ------------------------------------------------------------------ launchers

#define DISPATCH(ctx, CALL)                       \
    do {                                          \
        if ((ctx)->cfg.dtype == HAWK_FP32) {      \
            using Cfg = CfgF32;                   \
            CALL;                                 \
        } else {                                  \
            using Cfg = CfgBF16;                  \
            CALL;                                 \
        }                                         \
    } while (0)

template <class Cfg> static const typename Cfg::WT* wptr(hawk_ctx* c, size_t blob_off) {
    return reinterpret_cast<const typename Cfg::WT*>(c->ws + c->off.blob + blob_off);
}

void launch_embed_rows(hawk_ctx* c, const RowMap& map, int M) {
    DISPATCH(c, (embed_rows_kernel<Cfg><<<M, 256, 0, c->stream>>>(
                    wsp<typename Cfg::AT>(c, c->off.x), wptr<Cfg>(c, c->w.E), map, wsp<int32_t>(c, c->off.grid),
                    wsp<int32_t>(c, c->off.draft), c->N, c->kmax + 1, c->d)));
}

void launch_cond_rows(hawk_ctx* c, int M) {
    size_t total = (size_t)M * c->d;
    DISPATCH(c, (cond_rows_kernel<Cfg><<<(unsigned)((total + 255) / 256), 256, 0, c->stream>>>(
                    wsp<typename Cfg::AT>(c, c->off.x), wsp<float>(c, c->off.cond), total)));
}

void launch_rmsnorm(hawk_ctx* c, size_t off_in, size_t in_stride, size_t off_gain, size_t off_out, int M,
                    bool for_gemm) {
    uint16_t *hi = nullptr, *lo = nullptr;
    if (for_gemm) presplit_planes(c, off_out, M, c->d, &hi, &lo);
    if (c->cfg.dtype == HAWK_BF16 && c->d % 4 == 0 && in_stride % 4 == 0 && off_in % 16 == 0 && off_out % 16 == 0 && (c->off.blob + off_gain) % 8 == 0 &&
        c->d <= 8192) {
        const float* X = wsp<float>(c, off_in);
        const uint16_t* g = reinterpret_cast<const uint16_t*>(c->ws + c->off.blob + off_gain);
        float* out = wsp<float>(c, off_out);
        if (c->d <= 2048)
            rmsnorm_rows_kernel<2><<<M, 256, 0, c->stream>>>(X, g, out, c->d, in_stride, c->cfg.rms_eps, hi, lo);
        else if (c->d <= 4096)
            rmsnorm_rows_kernel<4><<<M, 256, 0, c->stream>>>(X, g, out, c->d, in_stride, c->cfg.rms_eps, hi, lo);
        else
            rmsnorm_rows_kernel<8><<<M, 256, 0, c->stream>>>(X, g, out, c->d, in_stride, c->cfg.rms_eps, hi, lo);
        return;
    }
    DISPATCH(c, (rmsnorm_kernel<Cfg><<<M, 256, 0, c->stream>>>(
                    wsp<typename Cfg::AT>(c, off_in), wptr<Cfg>(c, off_gain), wsp<typename Cfg::AT>(c, off_out),
                    c->d, in_stride, c->cfg.rms_eps, hi, lo)));
}

void launch_gemm(hawk_ctx* c, size_t off_a, int lda, size_t w_off, int N, int K, size_t off_y, int ldy,
                 int M, bool accumulate, bool out_f32) {
    if (launch_gemm_mfma(c, off_a, lda, w_off, N, K, off_y, ldy, M, accumulate)) return;
    constexpr int RT = 8;
    dim3 grid((N + 3) / 4, (M + RT - 1) / RT);
    if (out_f32) {
        DISPATCH(c, (gemm_rows_kernel<Cfg, RT, float><<<grid, 256, 0, c->stream>>>(
                        wsp<typename Cfg::AT>(c, off_a), lda, wptr<Cfg>(c, w_off), N, K, wsp<float>(c, off_y), ldy,
                        M, accumulate ? 1 : 0)));
    } else {
        DISPATCH(c, (gemm_rows_kernel<Cfg, RT, typename Cfg::AT><<<grid, 256, 0, c->stream>>>(
                        wsp<typename Cfg::AT>(c, off_a), lda, wptr<Cfg>(c, w_off), N, K,
                        wsp<typename Cfg::AT>(c, off_y), ldy, M, accumulate ? 1 : 0)));
    }
}

void launch_rope_append(hawk_ctx* c, const RowMap& map, int layer, int M) {
    DISPATCH(c, (rope_append_kernel<Cfg><<<M, 256, 0, c->stream>>>(
                    wsp<typename Cfg::AT>(c, c->off.qkv), wsp<typename Cfg::KT>(c, c->off.kc),
                    wsp<typename Cfg::KT>(c, c->off.vc), map, wsp<double>(c, c->off.inv_freq), layer, c->d, c->hd,
                    c->Smax, c->Tmax)));
}

// Step rows of a bf16 context go through attention_rows_kernel, which also does the rotary step
// and the cache append of its rows.
static size_t attention_rows_lds(const hawk_ctx* c) {
    return ((size_t)8 * c->hd + (size_t)c->Tmax * 8 + (size_t)4 * 8 * c->hd) * sizeof(float);
}
bool attention_does_rope(const hawk_ctx* c, const RowMap& map) {
    const int cpr = c->hd / 8;
    return c->cfg.dtype == HAWK_BF16 && map.mode == 1 && map.rows_per_seq <= 8 && (cpr == 8 || cpr == 16) &&
           attention_rows_lds(c) <= 60 * 1024;
}

void launch_attention(hawk_ctx* c, const RowMap& map, int layer, int M) {
    if (attention_does_rope(c, map)) {
        const size_t lds = attention_rows_lds(c);
        {
            dim3 grid(M / map.rows_per_seq, c->H);
            uint16_t *hi = nullptr, *lo = nullptr;
            presplit_planes(c, c->off.o, M, c->d, &hi, &lo);   // the Wo GEMM reads the result next
#define HAWK_ATTN_ROWS(RMV, NRV)                                                                       \
    attention_rows_kernel<RMV, NRV><<<grid, 256, lds, c->stream>>>(                                    \
        wsp<float>(c, c->off.qkv), wsp<_Float16>(c, c->off.kc), wsp<_Float16>(c, c->off.vc),           \
        wsp<float>(c, c->off.o), map, wsp<double>(c, c->off.inv_freq), layer, c->d, c->hd, c->Smax, c->Tmax, hi, lo)
            if (map.rows_per_seq <= 2) HAWK_ATTN_ROWS(4, 2);
            else if (map.rows_per_seq <= 4) HAWK_ATTN_ROWS(4, 4);
            else if (map.rows_per_seq <= 6) HAWK_ATTN_ROWS(8, 6);
            else HAWK_ATTN_ROWS(8, 8);
#undef HAWK_ATTN_ROWS
            return;
        }
    }
    dim3 grid(c->H, M);
    uint16_t *hi = nullptr, *lo = nullptr;
    if (map.mode == 2) presplit_planes(c, c->off.o, M, c->d, &hi, &lo);   // tree rows: the Wo product reads the result next
    DISPATCH(c, (attention_kernel<Cfg><<<grid, 256, (size_t)(c->Tmax + c->hd + 256) * sizeof(typename Cfg::AT),
                                         c->stream>>>(
                    wsp<typename Cfg::AT>(c, c->off.qkv), wsp<typename Cfg::KT>(c, c->off.kc),
                    wsp<typename Cfg::KT>(c, c->off.vc), wsp<typename Cfg::AT>(c, c->off.o), map, layer, c->d, c->hd,
                    c->Smax, c->Tmax, hi, lo)));
}

void launch_swiglu(hawk_ctx* c, int M) {
    size_t total = (size_t)M * c->m;
    uint16_t *hi = nullptr, *lo = nullptr;
    presplit_planes(c, c->off.u, M, c->m, &hi, &lo);   // the W2 GEMM reads the result next
    DISPATCH(c, (swiglu_kernel<Cfg><<<(unsigned)((total + 255) / 256), 256, 0, c->stream>>>(
                    wsp<typename Cfg::AT>(c, c->off.u), c->m, total, hi, lo)));
}

void launch_draft_input(hawk_ctx* c, int i) {
    // draft i writes its head output to g1 (i odd) / g0 (i even); draft i > 1 reads draft i-1's
    size_t prev = (i == 1) ? c->off.hprev : (((i - 1) & 1) ? c->off.g1 : c->off.g0);
    DISPATCH(c, (draft_input_kernel<Cfg><<<c->S, 256, 0, c->stream>>>(
                    wsp<typename Cfg::AT>(c, c->off.din), wsp<typename Cfg::AT>(c, prev), wptr<Cfg>(c, c->w.E),
                    wsp<int32_t>(c, c->off.n), wsp<int32_t>(c, c->off.k_eff), wsp<int32_t>(c, c->off.grid),
                    wsp<int32_t>(c, c->off.draft), i, c->B, c->N, c->gw, c->kmax + 1, c->d)));
}

void launch_keep_hprev_prefill(hawk_ctx* c) {
    DISPATCH(c, (keep_hprev_prefill_kernel<Cfg><<<c->S, 256, 0, c->stream>>>(
                    wsp<typename Cfg::AT>(c, c->off.hprev), wsp<typename Cfg::AT>(c, c->off.x), c->C, c->d)));
}

}  // namespace hawk
