// Spatial drafting structures (Method, "Dual Direction Drafting Heads", "Spatial Sampling Pool";
// appendix "Draft Heads Structure and Memory Overhead"): the dual-direction heads on the MFMA
// GEMM kernels, the speculation cache as a ring per (column, depth) in device memory, and the
// gather of a position's sampling pool.  No context: every entry point takes device pointers.
#include "hawk_internal.h"

namespace hawk {

namespace {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

// G[(r, j)] = h[r] + silu(Y[r][j d .. j d + d)), written as the two bf16 planes the output-layer
// GEMM reads (row r * n_heads + j, so that the logits come out as [rows][n_heads][V_s]) and, if
// asked for, as fp32.  One thread per four features.
__global__ void head_act_kernel(const float* h, const float* Y, int rows, int n_heads, int d, uint16_t* ghi,
                                uint16_t* glo, float* g_out) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int d4 = d / 4;
    if (i >= (size_t)rows * n_heads * d4) return;
    const size_t rj = i / d4;                 // r * n_heads + j
    const int f = (int)(i - rj * d4) * 4;
    const size_t r = rj / n_heads;
    const float4 x = *reinterpret_cast<const float4*>(h + r * d + f);
    const float4 y = *reinterpret_cast<const float4*>(Y + rj * d + f);   // Y is [rows][n_heads * d]
    float4 g;
    g.x = x.x + y.x / (1.0f + expf(-y.x));
    g.y = x.y + y.y / (1.0f + expf(-y.y));
    g.z = x.z + y.z / (1.0f + expf(-y.z));
    g.w = x.w + y.w / (1.0f + expf(-y.w));
    unsigned h0, h1, h2, h3, l0, l1, l2, l3;
    bf16_split(g.x, h0, l0);
    bf16_split(g.y, h1, l1);
    bf16_split(g.z, h2, l2);
    bf16_split(g.w, h3, l3);
    *reinterpret_cast<uint2*>(ghi + rj * d + f) = make_uint2(h0 | (h1 << 16), h2 | (h3 << 16));
    *reinterpret_cast<uint2*>(glo + rj * d + f) = make_uint2(l0 | (l1 << 16), l2 | (l3 << 16));
    if (g_out) *reinterpret_cast<float4*>(g_out + rj * d + f) = g;
}

// ---- speculation cache ----
// A prediction of depth dep for the position (row, col) waits in slot
//     col * S + dep (dep - 1) / 2 + row % dep,   S = VSD (VSD + 1) / 2:
// of one column and one depth at most dep predictions are outstanding at a time (those for the dep
// rows below the row being decoded), so a ring of dep slots holds them, and the rings of all
// depths and columns add up to the IW * VSD * (VSD + 1) / 2 entries the method names.  tag[slot] is
// the position the entry points to, -1 if none: a reader takes an entry only if the tag is the
// position it asks for.
struct CacheView {
    int32_t* tag;
    float* rows;
    int IW, VSD, S, Vs;
};

__host__ __device__ inline int slot_of(int IW, int S, int pos, int dep) {
    const int row = pos / IW, col = pos - row * IW;
    return col * S + dep * (dep - 1) / 2 + row % dep;
}

inline CacheView view(void* cache, int IW, int VSD, int Vs) {
    CacheView v;
    v.IW = IW; v.VSD = VSD; v.S = VSD * (VSD + 1) / 2; v.Vs = Vs;
    v.tag = static_cast<int32_t*>(cache);
    v.rows = reinterpret_cast<float*>(static_cast<char*>(cache) + align_up((size_t)IW * v.S * sizeof(int32_t)));
    return v;
}

__global__ void cache_reset_kernel(int32_t* tag, int slots) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < slots) tag[i] = -1;
}

__device__ __forceinline__ void copy_row(const float* src, float* dst, int n) {
    if (((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 15) == 0 && n % 4 == 0) {
        for (int e = threadIdx.x; e < n / 4; e += blockDim.x)
            reinterpret_cast<float4*>(dst)[e] = reinterpret_cast<const float4*>(src)[e];
    } else {
        for (int e = threadIdx.x; e < n; e += blockDim.x) dst[e] = src[e];
    }
}

// Block (dep - 1, r): the hidden state that predicted pos[r] also predicted pos[r] + dep * IW.
__global__ __launch_bounds__(256) void cache_push_kernel(CacheView c, int n_pos, const int32_t* pos, const float* q_vert,
                                                         size_t row_stride) {
    const int dep = blockIdx.x + 1, r = blockIdx.y;
    const int T = pos[r];
    if (T < 0 || T >= n_pos) return;
    const int t = T + dep * c.IW;
    if (t >= n_pos) return;   // below the image
    const int slot = slot_of(c.IW, c.S, t, dep);
    copy_row(q_vert + r * row_stride + (size_t)(dep - 1) * c.Vs, c.rows + (size_t)slot * c.Vs, c.Vs);
    if (threadIdx.x == 0) c.tag[slot] = t;
}

// Block (k, i): member k of the pool at target[i]; k < VSD is the cached prediction of depth and
// row distance k + 1, k == VSD the horizontal proposal.  Members that exist are packed to the front
// in that order.
__global__ __launch_bounds__(256) void pool_kernel(CacheView c, int n_pos, const int32_t* target, const float* q_horiz,
                                                   size_t horiz_stride, float* pool_logits, int32_t* pool_m,
                                                   int32_t* pool_delta) {
    const int k = blockIdx.x, i = blockIdx.y, m_max = c.VSD + 1;
    const int t = target[i];
    if (t < 0 || t >= n_pos) {
        if (k == c.VSD && threadIdx.x == 0) {
            pool_m[i] = 0;
            for (int j = 0; j < m_max; ++j) pool_delta[(size_t)i * m_max + j] = -1;
        }
        return;
    }
    int before = 0;          // members in front of this one
    bool mine = k == c.VSD;
    for (int dv = 1; dv <= min(k + 1, c.VSD); ++dv) {
        const bool have = c.tag[slot_of(c.IW, c.S, t, dv)] == t;
        if (dv == k + 1) mine = have;
        else before += have ? 1 : 0;
    }
    if (k == c.VSD) {
        if (threadIdx.x == 0) {
            pool_m[i] = before + 1;
            pool_delta[(size_t)i * m_max + before] = 0;
            for (int j = before + 1; j < m_max; ++j) pool_delta[(size_t)i * m_max + j] = -1;
        }
        copy_row(q_horiz + i * horiz_stride, pool_logits + ((size_t)i * m_max + before) * c.Vs, c.Vs);
        return;
    }
    if (!mine) return;
    if (threadIdx.x == 0) pool_delta[(size_t)i * m_max + before] = k + 1;
    copy_row(c.rows + (size_t)slot_of(c.IW, c.S, t, k + 1) * c.Vs, pool_logits + ((size_t)i * m_max + before) * c.Vs, c.Vs);
}

bool cache_args_ok(int IW, int IH, int VSD, int Vs) {
    return IW >= 1 && IH >= 1 && VSD >= 1 && VSD <= 16 && Vs >= 1 && (long)IW * IH < (1L << 30);
}

}  // namespace

size_t spatial_heads_workspace_bytes(int rows, int n_heads, int d) {
    const size_t M = (size_t)rows * n_heads;
    return align_up(M * d * sizeof(float)) + align_up(2 * (size_t)rows * d * 2) + align_up(2 * M * d * 2);
}

int launch_spatial_heads(const float* h, const uint16_t* W_heads, const uint16_t* W_out, int rows, int n_heads, int d,
                         int Vs, float* q_logits, float* g_out, void* workspace, size_t workspace_bytes,
                         hipStream_t stream) {
    if (d % 64 || Vs % 16) return HAWK_EINVAL;
    if (!workspace || workspace_bytes < spatial_heads_workspace_bytes(rows, n_heads, d)) return HAWK_EINVAL;
    if ((reinterpret_cast<uintptr_t>(workspace) | reinterpret_cast<uintptr_t>(h) | reinterpret_cast<uintptr_t>(q_logits) |
         reinterpret_cast<uintptr_t>(g_out) | reinterpret_cast<uintptr_t>(W_heads) | reinterpret_cast<uintptr_t>(W_out)) & 15)
        return HAWK_EINVAL;
    const int M = rows * n_heads;
    char* w = static_cast<char*>(workspace);
    float* Y = reinterpret_cast<float*>(w);
    w += align_up((size_t)M * d * sizeof(float));
    uint16_t* hplanes = reinterpret_cast<uint16_t*>(w);
    w += align_up(2 * (size_t)rows * d * 2);
    uint16_t* gplanes = reinterpret_cast<uint16_t*>(w);
    // every head's linear layer in one product, Y[r][j d + f] = (W_j h_r)[f], with the residual and
    // the activation in its epilogue where the shape allows (the workspace's Y then holds g)
    if (!gemm_rows_heads(stream, h, rows, d, W_heads, n_heads, g_out ? g_out : Y, hplanes, gplanes)) {
        if (!gemm_rows_bf16(stream, h, d, rows, d, W_heads, n_heads * d, Y, n_heads * d, hplanes)) return HAWK_EINVAL;
        const size_t total = (size_t)M * (d / 4);
        head_act_kernel<<<(unsigned)((total + 255) / 256), 256, 0, stream>>>(h, Y, rows, n_heads, d, gplanes,
                                                                            gplanes + (size_t)M * d, g_out);
    }
    // the shared output layer over all (row, head) pairs
    if (!gemm_rows_bf16(stream, nullptr, d, M, d, W_out, Vs, q_logits, Vs, gplanes)) return HAWK_EINVAL;
    return hipGetLastError() == hipSuccess ? HAWK_OK : HAWK_EDEVICE;
}

size_t spec_cache_bytes(int IW, int VSD, int Vs) {
    const size_t slots = (size_t)IW * VSD * (VSD + 1) / 2;
    return align_up(slots * sizeof(int32_t)) + slots * (size_t)Vs * sizeof(float);
}

int spec_cache_slot(int IW, int VSD, int pos, int depth) {
    if (IW < 1 || VSD < 1 || pos < 0 || depth < 1 || depth > VSD) return -1;
    return slot_of(IW, VSD * (VSD + 1) / 2, pos, depth);
}

int launch_spec_cache_reset(void* cache, int IW, int VSD, int Vs, hipStream_t stream) {
    if (!cache || !cache_args_ok(IW, 1, VSD, Vs)) return HAWK_EINVAL;
    const CacheView c = view(cache, IW, VSD, Vs);
    const int slots = IW * c.S;
    cache_reset_kernel<<<(slots + 255) / 256, 256, 0, stream>>>(c.tag, slots);
    return hipGetLastError() == hipSuccess ? HAWK_OK : HAWK_EDEVICE;
}

int launch_spec_cache_push(void* cache, int IW, int IH, int VSD, int Vs, const int32_t* pos, const float* q_vert,
                           size_t row_stride, int rows, hipStream_t stream) {
    if (!cache || !pos || !q_vert || !cache_args_ok(IW, IH, VSD, Vs) || rows < 0 || rows > IW) return HAWK_EINVAL;
    if (row_stride < (size_t)VSD * Vs) return HAWK_EINVAL;
    if (rows == 0) return HAWK_OK;
    cache_push_kernel<<<dim3(VSD, rows), 256, 0, stream>>>(view(cache, IW, VSD, Vs), IW * IH, pos, q_vert, row_stride);
    return hipGetLastError() == hipSuccess ? HAWK_OK : HAWK_EDEVICE;
}

int launch_spec_pool(const void* cache, int IW, int IH, int VSD, int Vs, const int32_t* target, const float* q_horiz,
                     size_t horiz_stride, int n, float* pool_logits, int32_t* pool_m, int32_t* pool_delta,
                     hipStream_t stream) {
    if (!cache || !target || !q_horiz || !pool_logits || !pool_m || !pool_delta || !cache_args_ok(IW, IH, VSD, Vs) || n < 0)
        return HAWK_EINVAL;
    if (horiz_stride < (size_t)Vs || n > 65535) return HAWK_EINVAL;
    if (n == 0) return HAWK_OK;
    pool_kernel<<<dim3(VSD + 1, n), 256, 0, stream>>>(view(const_cast<void*>(cache), IW, VSD, Vs), IW * IH, target, q_horiz,
                                                     horiz_stride, pool_logits, pool_m, pool_delta);
    return hipGetLastError() == hipSuccess ? HAWK_OK : HAWK_EDEVICE;
}

}  // namespace hawk
