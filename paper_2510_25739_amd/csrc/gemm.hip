// GEMMs of the one-kernel-per-operation path on the MFMA units, bf16 weights:
// Y[M][N] (+)= A[M][K] * W[N][K]^T.
//
// The fp32 activations enter as two bf16 planes, hi and lo (two MFMAs per tile: fp32-accurate
// activations); the kernel that produces a GEMM's input writes them, or split_rows_kernel does.
// The weights are read from a tile-major copy made when the blob is loaded (pack_tiles_kernel):
// 16 x 32 tiles of 1 KB in MFMA A-operand order, so that a wave's request is one contiguous
// kilobyte instead of 64-byte pieces of 16 rows (row-major weights still work, at about half the
// bandwidth).
//
// More than 16 rows (several prompts, guidance doubling, the prefill) - gemm_mfma_kernel: here
// every weight byte meets tens to hundreds of rows, a real contraction.
//   - a workgroup of four waves computes a tile of 16*SR*2 output features x 16*CT*2 rows: the
//     waves sit 2 x 2 over the tile, each holds SR x CT accumulators of v_mfma_f32_16x16x32_bf16;
//   - weight tiles go straight from global memory into VGPRs; the activation planes of the tile's
//     rows go through LDS (padded rows, double-buffered, 64 k per stage) because all four waves
//     read them;
//   - D stages are in flight per workgroup, held in a register ring, and the barrier between
//     stages orders LDS traffic only, so a stage costs its arithmetic and not a memory round trip;
//   - per k-step a wave issues 2*CT LDS reads for 2*SR*CT MFMAs.
// Up to 16 rows - gemv_mfma_kernel: weight streaming with a sliver of arithmetic; waves work
// alone, no LDS staging and no barrier in the loop (see there).
#include "hawk_internal.h"

namespace hawk {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned v4u __attribute__((ext_vector_type(4)));

constexpr int kKC = 64;          // k per LDS stage (two MFMA k-steps)
constexpr int kLdsK = kKC + 8;   // padded row length in halves

// Workgroup barrier that orders LDS traffic only: __syncthreads() also waits for every global
// load in flight, which would end the prefetch of the coming stages at each k-stage.
__device__ __forceinline__ void lds_barrier() {
    __atomic_signal_fence(__ATOMIC_SEQ_CST);
    __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0); vmcnt and expcnt left alone
    __builtin_amdgcn_s_barrier();
    __atomic_signal_fence(__ATOMIC_SEQ_CST);
}

// Tile-major copy of W[N][K] (N % 16 == 0, K % 32 == 0): tile (strip s, k-tile kt) is the 1 KB
// block number s * (K / 32) + kt; inside it lane l of a wave owns bytes 16 l .. 16 l + 15 = row
// s * 16 + l % 16, columns kt * 32 + (l / 16) * 8 .. + 7: one MFMA A operand per tile.
// pairs > 0 (W1|W3, pairs = m): strip s holds W1 rows 8 s .. 8 s + 7 and the matching W3 rows
// interleaved (row 2 j = W1 row 8 s + j, row 2 j + 1 = W3 row 8 s + j), so that an MFMA result lane
// holds both halves of a SwiGLU pair.
__global__ void pack_tiles_kernel(const uint16_t* W, int K, v4u* dst, size_t total, int pairs) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total) return;
    const int lane = (int)(i & 63), r = lane & 15;
    const size_t tile = i >> 6, kts = (size_t)K / 32, s = tile / kts, kt = tile - s * kts;
    const size_t row = pairs ? (size_t)(r & 1) * pairs + s * 8 + (r >> 1) : s * 16 + r;
    dst[i] = *reinterpret_cast<const v4u*>(W + row * (size_t)K + kt * 32 + (lane >> 4) * 8);
}

// SwiGLU of an MFMA result lane of a pair-interleaved W1|W3 tile: v = (a0, b0, a1, b1) -> two
// hidden features; writes them as fp32 into U (row stride ldy) and as bf16 hi / lo into the planes
// of the GEMM that follows (row stride om).
__device__ __forceinline__ void swiglu_store(f32x4 v, float* U, int ldy, uint16_t* ohi, uint16_t* olo, int om, int row,
                                             int f0) {
    const float h0 = v[0] / (1.0f + expf(-v[0])) * v[1], h1 = v[2] / (1.0f + expf(-v[2])) * v[3];
    *reinterpret_cast<float2*>(U + (size_t)row * ldy + f0) = make_float2(h0, h1);
    unsigned a0, b0, a1, b1;
    bf16_split(h0, a0, b0);
    bf16_split(h1, a1, b1);
    *reinterpret_cast<unsigned*>(ohi + (size_t)row * om + f0) = a0 | (a1 << 16);
    *reinterpret_cast<unsigned*>(olo + (size_t)row * om + f0) = b0 | (b1 << 16);
}

// hi[r][j], lo[r][j] = bf16 split of A[r * lda + j], r < M, j < K (K % 4 == 0).
__global__ void split_rows_kernel(const float* A, int lda, int K, uint16_t* hi, uint16_t* lo, size_t total4) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total4) return;
    const int k4 = K / 4;
    const size_t r = i / k4;
    const int j = (int)(i - r * k4) * 4;
    const float4 v = *reinterpret_cast<const float4*>(A + r * lda + j);
    unsigned h0, h1, h2, h3, l0, l1, l2, l3;
    bf16_split(v.x, h0, l0);
    bf16_split(v.y, h1, l1);
    bf16_split(v.z, h2, l2);
    bf16_split(v.w, h3, l3);
    *reinterpret_cast<uint2*>(hi + r * K + j) = make_uint2(h0 | (h1 << 16), h2 | (h3 << 16));
    *reinterpret_cast<uint2*>(lo + r * K + j) = make_uint2(l0 | (l1 << 16), l2 | (l3 << 16));
}

// SR: 16-feature strips per wave, CT: 16-row tiles per wave, D: stages (64 k each) in flight.
// Tile = (32 SR) features x (32 CT) rows.
template <int SR, int CT, int D>
__global__ __launch_bounds__(256) void gemm_mfma_kernel(const uint16_t* __restrict__ hi, const uint16_t* __restrict__ lo,
                                                        const uint16_t* __restrict__ W, int packed, int N, int K,
                                                        float* Y, int ldy, int M, int accumulate, uint16_t* ohi,
                                                        uint16_t* olo, int om) {
    constexpr int BM = 32 * CT, BN = 32 * SR;
    constexpr int CHUNKS = 2 * BM * (kKC / 8);       // 16-byte chunks of one stage (both planes)
    constexpr int PER_T = (CHUNKS + 255) / 256;
    __shared__ __attribute__((aligned(16))) uint16_t lds[2][2][BM][kLdsK];   // [buffer][plane][row][k]
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int wn = wave >> 1, wm = wave & 1;                     // wave position over (features, rows)
    const int n0 = blockIdx.x * BN + wn * 16 * SR, m0 = blockIdx.y * BM;
    const int r16 = lane & 15, kg = lane >> 4;
    const int nk = K / kKC, it0 = 0;

    static_assert(CHUNKS % 256 == 0, "a stage is a whole number of 16-byte chunks per thread");

    // weights: W is either row-major [N][K] or the tile-major copy (see pack_tiles_kernel); per
    // strip a base pointer for this lane and a stride per 32-k tile
    const size_t wstride = packed ? 512 : 32;
    const uint16_t* wbase[SR];
#pragma unroll
    for (int t = 0; t < SR; ++t) {
        const int strip = min((n0 + t * 16) / 16, N / 16 - 1);   // strips past the end repeat the last (never stored)
        wbase[t] = packed ? W + ((size_t)strip * (K / 32)) * 512 + lane * 8 : W + (size_t)(strip * 16 + r16) * K + kg * 8;
    }
    struct Stage { v4u b[PER_T]; v4u w[SR][2]; };
    // Everything of stage `it` that comes from global memory: the tile rows' activation planes
    // (chunk q -> plane, row, 8-k group) and the wave's weight tiles (SR strips x 2 k-steps).
    // Every lane always loads (rows and features past the end are clamped to the last one; what
    // they produce is never stored), and the loop below never branches around a load: only then
    // can the waits for an old stage be counted past the younger requests behind it.
    auto load_stage = [&](int it, Stage& s) {
        const size_t k0 = (size_t)(it0 + min(it, nk - 1)) * kKC;
#pragma unroll
        for (int i = 0; i < PER_T; ++i) {
            const int q = i * 256 + threadIdx.x;
            const int pl = q / (BM * (kKC / 8)), rem = q - pl * (BM * (kKC / 8));
            const int row = rem / (kKC / 8), g = rem - row * (kKC / 8);
            const uint16_t* src = (pl ? lo : hi) + (size_t)min(m0 + row, M - 1) * K + k0 + g * 8;
            s.b[i] = *reinterpret_cast<const v4u*>(src);
        }
#pragma unroll
        for (int t = 0; t < SR; ++t) {
#pragma unroll
            for (int ks = 0; ks < 2; ++ks)
                s.w[t][ks] = *reinterpret_cast<const v4u*>(wbase[t] + (k0 / 32 + ks) * wstride);
        }
    };
    auto store_stage = [&](int buf, const Stage& s) {
#pragma unroll
        for (int i = 0; i < PER_T; ++i) {
            const int q = i * 256 + threadIdx.x;
            const int pl = q / (BM * (kKC / 8)), rem = q - pl * (BM * (kKC / 8));
            const int row = rem / (kKC / 8), g = rem - row * (kKC / 8);
            *reinterpret_cast<v4u*>(&lds[buf][pl][row][g * 8]) = s.b[i];
        }
    };

    f32x4 acc[SR][CT], acl[SR][CT];
#pragma unroll
    for (int s = 0; s < SR; ++s)
#pragma unroll
        for (int t = 0; t < CT; ++t) {
            acc[s][t] = (f32x4){0.f, 0.f, 0.f, 0.f};
            acl[s][t] = (f32x4){0.f, 0.f, 0.f, 0.f};
        }
    // one k-stage: weights from the ring slot, activations from LDS buffer `buf`
    auto compute = [&](int buf, const Stage& st) {
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            v4u bh[CT], bl[CT];
#pragma unroll
            for (int t = 0; t < CT; ++t) {
                const int row = wm * 16 * CT + t * 16 + r16;
                bh[t] = *reinterpret_cast<const v4u*>(&lds[buf][0][row][ks * 32 + kg * 8]);
                bl[t] = *reinterpret_cast<const v4u*>(&lds[buf][1][row][ks * 32 + kg * 8]);
            }
#pragma unroll
            for (int s = 0; s < SR; ++s) {
                const bf16x8 a = __builtin_bit_cast(bf16x8, st.w[s][ks]);
#pragma unroll
                for (int t = 0; t < CT; ++t) {
                    acc[s][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, __builtin_bit_cast(bf16x8, bh[t]), acc[s][t], 0, 0, 0);
                    acl[s][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, __builtin_bit_cast(bf16x8, bl[t]), acl[s][t], 0, 0, 0);
                }
            }
        }
    };
    Stage ring[D];   // stage s lives in slot s % D from its request until its last use
#pragma unroll
    for (int j = 0; j < D; ++j) load_stage(j, ring[j]);
    store_stage(0, ring[0]);
    lds_barrier();
    int it = 0;
    for (; it + D <= nk; it += D) {
#pragma unroll
        for (int j = 0; j < D; ++j) {
            const int buf = (it + j) & 1;
            compute(buf, ring[j]);
            store_stage(buf ^ 1, ring[(j + 1) % D]);   // stage it + j + 1, requested D - 1 stages ago
            load_stage(it + j + D, ring[j]);
            lds_barrier();
        }
    }
#pragma unroll
    for (int j = 0; j < D - 1; ++j) {   // the last nk % D stages: nothing left to request
        if (it + j < nk) {
            const int buf = (it + j) & 1;
            compute(buf, ring[j]);
            store_stage(buf ^ 1, ring[j + 1]);
            lds_barrier();
        }
    }
    // lane holds features n0 + s*16 + 4*kg .. +3 of row m0 + wm*16*CT + t*16 + r16
#pragma unroll
    for (int s = 0; s < SR; ++s)
#pragma unroll
        for (int t = 0; t < CT; ++t) {
            const int m = m0 + wm * 16 * CT + t * 16 + r16, n = n0 + s * 16 + 4 * kg;
            if (m < M && n < N) {
                float* dst = Y + (size_t)m * ldy + n;
                f32x4 v = acc[s][t] + acl[s][t];
                if (om > 0) {   // pair-interleaved W1|W3: n / 2 is the first of the lane's two hidden features
                    swiglu_store(v, Y, ldy, ohi, olo, om, m, n / 2);
                    continue;
                }
                if (accumulate) {
                    const float4 old = *reinterpret_cast<const float4*>(dst);
                    v += (f32x4){old.x, old.y, old.z, old.w};
                }
                *reinterpret_cast<float4*>(dst) = make_float4(v[0], v[1], v[2], v[3]);
            }
        }
}

// At most 16 rows: Y[M][N] (+)= A W^T is weight streaming with a sliver of arithmetic, and staging
// the rows through LDS with a barrier per k-stage would cost more than the streaming itself.  Here
// a wave works alone: it owns SR strips of 16 features over a quarter of K, loads weight tiles
// (A operand) and the rows' bf16 planes (B operand, from L2) straight into registers in MFMA
// layout, D k-steps ahead, with no barrier in the loop; the four waves of a workgroup - the four
// K quarters of the same strips - add their tiles through LDS at the end.  K % 128 == 0.
template <int SR, int D>
__global__ __launch_bounds__(256) void gemv_mfma_kernel(const uint16_t* __restrict__ hi, const uint16_t* __restrict__ lo,
                                                        const uint16_t* __restrict__ W, int packed, int N, int K,
                                                        float* Y, int ldy, int M, int accumulate, uint16_t* ohi,
                                                        uint16_t* olo, int om, const float* resid) {
    __shared__ f32x4 red[3][SR][64];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int r16 = lane & 15, kg = lane >> 4;
    const int n0 = blockIdx.x * 16 * SR;
    const int nk = K / 128;                               // k-steps (32 k each) of this wave's quarter
    const size_t kbase = (size_t)wave * (K / 4) + kg * 8;
    // weights row-major or tile-major (see pack_tiles_kernel): base pointer per strip, stride per k-step
    const size_t wstride = packed ? 512 : 32;
    const uint16_t* wp[SR];
#pragma unroll
    for (int s = 0; s < SR; ++s) {
        const int strip = min(n0 / 16 + s, N / 16 - 1);   // strips past the end repeat the last (never stored)
        wp[s] = packed ? W + ((size_t)strip * (K / 32) + (size_t)wave * (K / 128)) * 512 + lane * 8
                       : W + (size_t)(strip * 16 + r16) * K + kbase;
    }
    const size_t arow = (size_t)min(r16, M - 1) * K + kbase;   // rows past the end repeat the last one (never stored)
    const uint16_t *hp = hi + arow, *lp = lo + arow;
    struct Step { v4u w[SR], bh, bl; };
    auto load = [&](int ks, Step& st) {
        const int kc = min(ks, nk - 1);          // requests past the end repeat the last step (unused)
        const int off = kc * 32;
#pragma unroll
        for (int s = 0; s < SR; ++s) st.w[s] = __builtin_nontemporal_load(reinterpret_cast<const v4u*>(wp[s] + kc * wstride));
        st.bh = *reinterpret_cast<const v4u*>(hp + off);
        st.bl = *reinterpret_cast<const v4u*>(lp + off);
    };
    f32x4 acc[SR], acl[SR];
#pragma unroll
    for (int s = 0; s < SR; ++s) {
        acc[s] = (f32x4){0.f, 0.f, 0.f, 0.f};
        acl[s] = (f32x4){0.f, 0.f, 0.f, 0.f};
    }
    auto fma_step = [&](const Step& st) {
#pragma unroll
        for (int s = 0; s < SR; ++s) {
            const bf16x8 a = __builtin_bit_cast(bf16x8, st.w[s]);
            acc[s] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, __builtin_bit_cast(bf16x8, st.bh), acc[s], 0, 0, 0);
            acl[s] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, __builtin_bit_cast(bf16x8, st.bl), acl[s], 0, 0, 0);
        }
    };
    Step ring[D];
#pragma unroll
    for (int j = 0; j < D; ++j) load(j, ring[j]);
    int ks = 0;
    for (; ks + D <= nk; ks += D) {
#pragma unroll
        for (int j = 0; j < D; ++j) {
            fma_step(ring[j]);
            load(ks + j + D, ring[j]);
        }
    }
#pragma unroll
    for (int j = 0; j < D - 1; ++j)
        if (ks + j < nk) fma_step(ring[j]);
    // lane holds features n0 + s*16 + 4*kg .. +3 of row r16
    if (wave > 0) {
#pragma unroll
        for (int s = 0; s < SR; ++s) red[wave - 1][s][lane] = acc[s] + acl[s];
    }
    __syncthreads();
    if (wave > 0) return;
#pragma unroll
    for (int s = 0; s < SR; ++s) {
        f32x4 v = (acc[s] + acl[s]) + red[0][s][lane] + (red[1][s][lane] + red[2][s][lane]);
        const int n = n0 + s * 16 + 4 * kg;
        if (r16 < M && n < N) {
            float* dst = Y + (size_t)r16 * ldy + n;
            if (om > 0) {   // pair-interleaved W1|W3
                swiglu_store(v, Y, ldy, ohi, olo, om, r16, n / 2);
                continue;
            }
            if (om < 0) {   // -om square blocks of K features (draft heads): g = a + silu(y) with a = resid[row],
                            // stored as row (row * blocks + block) of Y ([M * blocks][K] fp32) and of the planes
                const int nb = -om, j = n / K, f = n - j * K;
                const float4 a = *reinterpret_cast<const float4*>(resid + (size_t)r16 * K + f);
                const float g0 = a.x + v[0] / (1.0f + expf(-v[0])), g1 = a.y + v[1] / (1.0f + expf(-v[1]));
                const float g2 = a.z + v[2] / (1.0f + expf(-v[2])), g3 = a.w + v[3] / (1.0f + expf(-v[3]));
                const size_t at = ((size_t)r16 * nb + j) * K + f;
                *reinterpret_cast<float4*>(Y + at) = make_float4(g0, g1, g2, g3);
                unsigned h0, h1, h2, h3, l0, l1, l2, l3;
                bf16_split(g0, h0, l0);
                bf16_split(g1, h1, l1);
                bf16_split(g2, h2, l2);
                bf16_split(g3, h3, l3);
                *reinterpret_cast<uint2*>(ohi + at) = make_uint2(h0 | (h1 << 16), h2 | (h3 << 16));
                *reinterpret_cast<uint2*>(olo + at) = make_uint2(l0 | (l1 << 16), l2 | (l3 << 16));
                continue;
            }
            if (accumulate) {
                const float4 old = *reinterpret_cast<const float4*>(dst);
                v += (f32x4){old.x, old.y, old.z, old.w};
            }
            *reinterpret_cast<float4*>(dst) = make_float4(v[0], v[1], v[2], v[3]);
        }
    }
}

}  // namespace

// Runs Y (+)= A W^T on the MFMA path if the shape allows; false: the caller uses the generic kernel.
static bool mfma_input_ok(const hawk_ctx* c, int M, int K) {
    return c->cfg.dtype == HAWK_BF16 && c->off.split && M >= 1 && K % kKC == 0 && (size_t)M * K * 4 <= c->split_bytes;
}

int gemm_pack_weights(hawk_ctx* c) {
    if (!c->off.gpack) return 0;
    for (int i = 0; i < c->n_gpk; ++i) {
        const auto& e = c->gpk[i];
        const size_t total = (size_t)e.N * e.K / 8;   // 16-byte chunks
        pack_tiles_kernel<<<(unsigned)((total + 255) / 256), 256, 0, c->stream>>>(
            reinterpret_cast<const uint16_t*>(c->ws + c->off.blob + e.blob_off), e.K,
            reinterpret_cast<v4u*>(c->ws + c->off.gpack + e.pack_off), total, e.pairs);
    }
    if (hipGetLastError() != hipSuccess) return -1;
    return hipStreamSynchronize(c->stream) == hipSuccess ? 0 : -1;
}

bool presplit_planes(hawk_ctx* c, size_t off_a, int M, int K, uint16_t** hi, uint16_t** lo) {
    if (!mfma_input_ok(c, M, K)) return false;
    *hi = wsp<uint16_t>(c, c->off.split);
    *lo = *hi + (size_t)M * K;
    c->presplit_off = off_a;
    c->presplit_M = M;
    c->presplit_K = K;
    c->presplit_buf = 0;
    return true;
}

// Tile choice and launch for Y (+)= A W^T with A given as its two bf16 planes.
static void launch_tiles(hipStream_t stream, const uint16_t* hi, const uint16_t* lo, const uint16_t* W, int packed, int N,
                         int K, float* Y, int ldy, int M, int acc, uint16_t* ohi, uint16_t* olo, int swiglu_m,
                         const float* resid = nullptr) {
    // The smallest tile that still gives every compute unit at most one workgroup: with so few
    // rows the kernel is bound by what one compute unit can stage and feed per k-stage, so the
    // work is spread as widely as one round of workgroups allows; larger grids than that only
    // re-read the activations more often.
    static const int cus = [] {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
        return n;
    }();
    auto tiles = [&](int bn, int bm) { return (long)((N + bn - 1) / bn) * ((M + bm - 1) / bm); };
#define HAWK_GEMM_TILE(SR, CT, D)                                                                      \
    do {                                                                                               \
        dim3 grid((N + 32 * SR - 1) / (32 * SR), (M + 32 * CT - 1) / (32 * CT), 1);                    \
        gemm_mfma_kernel<SR, CT, D><<<grid, 256, 0, stream>>>(hi, lo, W, packed, N, K, Y, ldy, M, acc, ohi, olo,    \
                                                                  swiglu_m);                            \
    } while (0)
    if (M <= 16 && K % 128 == 0) {   // a sliver of rows: barrier-free weight streaming, one wave per K quarter
        // Strips per workgroup and k-steps in flight, from timings over weights that do not fit the
        // last-level cache (7B and XL shapes, 12 rows): 64 features per workgroup when that gives one
        // round of workgroups over most of the chip, 32 when there are enough strips to fill it,
        // else 16 with a deeper ring (a shallower one again for long K).
#define HAWK_GEMV(SR, D) gemv_mfma_kernel<SR, D><<<(N + 16 * SR - 1) / (16 * SR), 256, 0, stream>>>(hi, lo, W, packed, N, K, Y, ldy, M, acc, ohi, olo, swiglu_m, resid)
        const long s64 = N / 64, s32 = N / 32;
        if (4 * s64 >= 3 * (long)cus && s64 <= (long)cus) HAWK_GEMV(4, 3);
        else if (5 * s32 >= 3 * (long)cus) HAWK_GEMV(2, 6);
        else if (K / 128 <= 32) HAWK_GEMV(1, 12);
        else HAWK_GEMV(1, 8);
#undef HAWK_GEMV
        return;
    }
    if (tiles(32, 32) <= cus) HAWK_GEMM_TILE(1, 1, 4);
    else if (tiles(32, 64) <= cus) HAWK_GEMM_TILE(1, 2, 4);
    else if (tiles(64, 64) <= cus) HAWK_GEMM_TILE(2, 2, 3);   // at equal area more features per tile: fewer LDS reads per MFMA
    else if (tiles(96, 64) <= cus) HAWK_GEMM_TILE(3, 2, 3);
    else HAWK_GEMM_TILE(4, 3, 2);
#undef HAWK_GEMM_TILE
}


// Common body: Y (+)= A W^T, or with swiglu_m > 0 the fused W1|W3 form (N = 2 swiglu_m).
static bool run_mfma(hawk_ctx* c, size_t off_a, int lda, size_t w_off, int N, int K, size_t off_y, int ldy, int M,
                     bool accumulate, int swiglu_m) {
    if (!mfma_input_ok(c, M, K) || N % 16 || ldy % 4 || lda % 4) {
        if (!swiglu_m) c->presplit_off = 0;
        return false;
    }
    const uint16_t* W = reinterpret_cast<const uint16_t*>(c->ws + c->off.blob + w_off);
    int packed = 0;
    if (c->off.gpack)
        for (int i = 0; i < c->n_gpk; ++i)
            if (c->gpk[i].blob_off == w_off && c->gpk[i].N == N && c->gpk[i].K == K && c->gpk[i].pairs == swiglu_m) {
                W = reinterpret_cast<const uint16_t*>(c->ws + c->off.gpack + c->gpk[i].pack_off);
                packed = 1;
                break;
            }
    if (swiglu_m && (!packed || !c->off.split2)) return false;   // the caller falls back to GEMM + SwiGLU kernel
    const bool presplit = c->presplit_off == off_a && c->presplit_M == M && c->presplit_K == K;
    c->presplit_off = 0;
    uint16_t* hi = wsp<uint16_t>(c, presplit && c->presplit_buf ? c->off.split2 : c->off.split);
    uint16_t* lo = hi + (size_t)M * K;
    if (!presplit) {
        const size_t total4 = (size_t)M * (K / 4);
        split_rows_kernel<<<(unsigned)((total4 + 255) / 256), 256, 0, c->stream>>>(wsp<float>(c, off_a), lda, K, hi, lo, total4);
    }
    float* Y = wsp<float>(c, off_y);
    uint16_t *ohi = nullptr, *olo = nullptr;
    if (swiglu_m) {   // the result's planes go to the second pair (the first is being read) and count as current
        ohi = wsp<uint16_t>(c, c->off.split2);
        olo = ohi + (size_t)M * swiglu_m;
        c->presplit_off = off_y;
        c->presplit_M = M;
        c->presplit_K = swiglu_m;
        c->presplit_buf = 1;
    }
    launch_tiles(c->stream, hi, lo, W, packed, N, K, Y, ldy, M, accumulate ? 1 : 0, ohi, olo, swiglu_m);
    return true;
}

bool gemm_rows_bf16(hipStream_t stream, const float* A, int lda, int M, int K, const uint16_t* W, int N, float* Y,
                    int ldy, uint16_t* planes) {
    if (M < 1 || K % kKC || N % 16 || ldy % 4 || lda % 4) return false;
    uint16_t *hi = planes, *lo = planes + (size_t)M * K;
    if (A) {
        const size_t total4 = (size_t)M * (K / 4);
        split_rows_kernel<<<(unsigned)((total4 + 255) / 256), 256, 0, stream>>>(A, lda, K, hi, lo, total4);
    }
    launch_tiles(stream, hi, lo, W, 0, N, K, Y, ldy, M, 0, nullptr, nullptr, 0);
    return true;
}

bool gemm_rows_heads(hipStream_t stream, const float* A, int M, int K, const uint16_t* W, int blocks, float* G,
                     uint16_t* planes_a, uint16_t* planes_g) {
    if (M < 1 || M > 16 || K % 128 || blocks < 1) return false;
    const size_t total4 = (size_t)M * (K / 4);
    split_rows_kernel<<<(unsigned)((total4 + 255) / 256), 256, 0, stream>>>(A, K, K, planes_a, planes_a + (size_t)M * K, total4);
    launch_tiles(stream, planes_a, planes_a + (size_t)M * K, W, 0, blocks * K, K, G, K, M, 0, planes_g,
                 planes_g + (size_t)M * blocks * K, -blocks, A);
    return true;
}

bool launch_gemm_mfma(hawk_ctx* c, size_t off_a, int lda, size_t w_off, int N, int K, size_t off_y, int ldy, int M,
                      bool accumulate) {
    return run_mfma(c, off_a, lda, w_off, N, K, off_y, ldy, M, accumulate, 0);
}

bool launch_gemm_swiglu(hawk_ctx* c, size_t off_a, int lda, size_t w13_off, int m, int K, size_t off_u, int M) {
    return run_mfma(c, off_a, lda, w13_off, 2 * m, K, off_u, 2 * m, M, false, m);
}

}  // namespace hawk
