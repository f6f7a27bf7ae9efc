// Weight-streaming verify pass: the whole target pass over the k+1 rows of every sequence
// (all layers + output projection) as ONE persistent kernel of 256 workgroups, one per CU.
//
// Why this shape (MI355X, measured): at batch 1 a layer of the XL model is 40 MB, i.e. ~5 us
// of HBM time, but it has five dependent matrix stages; a kernel boundary costs ~6 us for an
// 8 MB kernel and a full HBM round trip ~1.5 us, so the stages must live in one kernel and the
// weights of stage p+1 must already be in flight while stage p synchronises.
//   - every matrix is pre-packed into 16x32 bf16 tiles laid out exactly as the A operand of
//     v_mfma_f32_16x16x32_bf16 (16 bytes per lane), in the order each wave consumes them;
//   - a workgroup owns whole 16-row output strips; its four compute waves split K four ways,
//     stream their tiles straight from HBM into VGPRs (no LDS staging of weights), and issue
//     the loads of their NEXT job right after the MFMAs of the current one, so that they land
//     while the grid barrier is being crossed;
//   - the k+1 activation rows are the B operand (columns 0..MR-1 of 16), staged in LDS as a
//     bf16 hi + lo pair (two MFMAs per tile: fp32-accurate activations at no HBM cost);
//   - two IO waves per workgroup do everything latency-bound: cross the barrier, fetch the
//     stage input with device-coherent loads, normalise, split, and later write the strip's
//     results; compute waves never wait on anything but their own weights;
//   - a grid barrier = arrival counters in 16 groups + top counter + replicated release word
//     (1.5 us measured; flat counters or all-to-all flags are 2-3x slower on 8 XCDs).
// Attention reads the fp16 KV cache with (head, chunk) jobs over all workgroups and a second
// small stage that merges the chunk partials.
#include <math.h>
#include <string.h>

#include <algorithm>
#include <vector>

#include "hawk_internal.h"

namespace hawk {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned long long u64;
typedef unsigned v4u __attribute__((ext_vector_type(4)));

constexpr int kCW = 4;                          // compute waves per workgroup
constexpr int kNIO = 2;                         // IO waves per workgroup
constexpr int kThreads = (kCW + kNIO) * 64;
constexpr int kTMax = 30;                       // tiles (1 KB each) a wave holds for one job
constexpr int kMaxStrips = 3;
constexpr int kGroups = 16, kReplicas = 8;      // barrier fan-in / release fan-out
constexpr unsigned kSpinLimit = 1u << 21;

// ------------------------------------------------------------------------- kernel parameters

struct SP {
    const uint4* wpack;
    u64 layer_tiles, kind_base[4], lm_base, wd_base;
    const int32_t* tab[K_NKIND];
    int32_t rounds[K_NKIND];
    const uint32_t* hasmask;  // per workgroup: bit kind (layer kinds), bit 8+r = LM round r
    const uint16_t* blob;
    u64 g1_off, g2_off, layer_bytes, gf_off;
    const float2* rope;
    _Float16* Kc;
    _Float16* Vc;
    float *X, *X2, *Q, *P, *O, *Hb, *logit_s;
    unsigned* bar;
    unsigned* err;
    const int32_t* n;
    const int32_t* k_eff;
    unsigned epoch0;
    int32_t L, d, H, m, Vs, S, B, C, RS, MR, NC, Smax, Tmax, Kp;
    float eps;
};

// ------------------------------------------------------------------------- device helpers

__device__ __forceinline__ float ld_f32(const float* p) {
    return __uint_as_float(__hip_atomic_load(reinterpret_cast<const unsigned*>(p), __ATOMIC_RELAXED,
                                             __HIP_MEMORY_SCOPE_AGENT));
}
__device__ __forceinline__ void st_f32(float* p, float v) {
    __hip_atomic_store(reinterpret_cast<unsigned*>(p), __float_as_uint(v), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float2 ld_f32x2(const float* p) {
    u64 v = __hip_atomic_load(reinterpret_cast<const u64*>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return make_float2(__uint_as_float((unsigned)v), __uint_as_float((unsigned)(v >> 32)));
}
__device__ __forceinline__ void st_f32x2(float* p, float a, float b) {
    u64 v = (u64)__float_as_uint(a) | ((u64)__float_as_uint(b) << 32);
    __hip_atomic_store(reinterpret_cast<u64*>(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint16_t bf16_rne(float f) {
    unsigned u = __float_as_uint(f);
    return (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
}
__device__ __forceinline__ float bf16_f32(unsigned b) { return __uint_as_float(b << 16); }
__device__ __forceinline__ float wsum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// Grid barrier.  Counters only ever grow (epochs continue across launches), so nothing is
// reset between kernels.  Waits are bounded: a workgroup that gives up raises *err and stops
// waiting for the rest of the kernel, so that every wave always terminates.
struct Barrier {
    unsigned* mem;
    unsigned* err;
    unsigned id;       // barriers completed so far (global count)
    unsigned first;    // id at kernel start
    bool dead;
    __device__ void arrive() {  // one lane of one wave per workgroup
        ++id;
        const unsigned g = blockIdx.x % kGroups, per = gridDim.x / kGroups;
        unsigned prev = __hip_atomic_fetch_add(mem + (size_t)g * 1024, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (prev + 1 == id * per) {
            unsigned t = __hip_atomic_fetch_add(mem + (size_t)kGroups * 1024, 1u, __ATOMIC_RELAXED,
                                                __HIP_MEMORY_SCOPE_AGENT);
            if (t + 1 == id * kGroups)
                for (int r = 0; r < kReplicas; ++r)
                    __hip_atomic_store(mem + (size_t)(kGroups + 1 + r) * 1024, id, __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    __device__ void wait() {  // whole wave; returns when barrier `id` has been released
        if (id == first || dead) return;
        const unsigned* rel = mem + (size_t)(kGroups + 1 + blockIdx.x % kReplicas) * 1024;
        for (unsigned spins = 0; spins < kSpinLimit; ++spins) {
            unsigned v = __hip_atomic_load(rel, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if ((int)(v - id) >= 0) return;
            if (__hip_atomic_load(err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u) break;
            __builtin_amdgcn_s_sleep(2);
        }
        dead = true;
        __hip_atomic_store(err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
};

struct Job {
    u64 tile0;       // first tile of wave 0 in wpack
    int nstrips;     // 0: no job
    int strip[kMaxStrips];
};

__device__ __forceinline__ Job load_job(const SP& p, int kind, int round, int layer) {
    const int32_t* e = p.tab[kind] + ((size_t)round * gridDim.x + blockIdx.x) * 4;
    Job j;
    j.nstrips = e[1];
    j.strip[0] = e[2] & 0xFFFF;
    j.strip[1] = (e[2] >> 16) & 0xFFFF;
    j.strip[2] = e[3] & 0xFFFF;
    u64 base = kind <= K_E ? (u64)layer * p.layer_tiles + p.kind_base[kind] : (kind == K_LM ? p.lm_base : p.wd_base);
    j.tile0 = base + (u64)(unsigned)e[0];
    return j;
}

// Issues the 16-byte loads of one wave's tiles of a job (nothing is waited for here).
__device__ __forceinline__ void issue_tiles(const SP& p, const Job& j, int tps, int wave, int lane, v4u (&w)[kTMax]) {
    const int nt = j.nstrips * tps;
    const v4u* src = reinterpret_cast<const v4u*>(p.wpack + (j.tile0 + (u64)wave * nt) * 64 + lane);
#pragma unroll
    for (int t = 0; t < kTMax; ++t)
        if (t < nt) {
            w[t] = __builtin_nontemporal_load(src + (size_t)t * 64);
        } else {
            w[t] = (v4u){0u, 0u, 0u, 0u};  // every slot is redefined: no value outlives its job
        }
}

// Stage input rows into LDS as bf16 hi / lo pairs: act[c][j] = split(src[c][j] * scale_c * gain_j).
// Row c is handled by IO wave (c mod kNIO).  NORM: RMS-normalise with the gain vector.
template <bool NORM, int KREG>
__device__ __forceinline__ void stage_rows(const float* src, int K, int MR, const uint16_t* gain, float eps, int io,
                                           int lane, uint16_t* act_hi, uint16_t* act_lo, int Kp) {
    for (int c = io; c < MR; c += kNIO) {
        float2 v[KREG];
        const float* row = src + (size_t)c * K;
#pragma unroll
        for (int i = 0; i < KREG; ++i) {
            int j = (i * 64 + lane) * 2;
            v[i] = j < K ? ld_f32x2(row + j) : make_float2(0.f, 0.f);
        }
        float r = 1.f;
        if (NORM) {
            float ss = 0.f;
#pragma unroll
            for (int i = 0; i < KREG; ++i) ss += v[i].x * v[i].x + v[i].y * v[i].y;
            ss = wsum(ss);
            r = 1.0f / sqrtf(ss / (float)K + eps);
        }
#pragma unroll
        for (int i = 0; i < KREG; ++i) {
            int j = (i * 64 + lane) * 2;
            if (j < K) {
                float a = v[i].x, b = v[i].y;
                if (NORM) {
                    unsigned g2 = *reinterpret_cast<const unsigned*>(gain + j);
                    a = a * r * bf16_f32(g2 & 0xFFFFu);
                    b = b * r * bf16_f32(g2 >> 16);
                }
                unsigned ha = bf16_rne(a), hb = bf16_rne(b);
                unsigned la = bf16_rne(a - bf16_f32(ha)), lb = bf16_rne(b - bf16_f32(hb));
                *reinterpret_cast<unsigned*>(act_hi + (size_t)c * Kp + j) = ha | (hb << 16);
                *reinterpret_cast<unsigned*>(act_lo + (size_t)c * Kp + j) = la | (lb << 16);
            }
        }
    }
}

// One wave's MFMAs of a job: strips x its K quarter, activations from LDS.  The B operand of
// a k-tile is shared by every strip of the job, and is fetched two k-tiles ahead.
template <int TPS>
__device__ __forceinline__ void mfma_job(const v4u (&w)[kTMax], int nstrips, int wave, int lane, int MR,
                                         const uint16_t* act_hi, const uint16_t* act_lo, int Kp, f32x4 (&acc)[kMaxStrips]) {
    constexpr int NS = kTMax / TPS < kMaxStrips ? kTMax / TPS : kMaxStrips;  // strips a job of this kind can have
    const int col = lane & 15, kg = lane >> 4;
    const bool live = col < MR;
    const uint16_t* bh_base = act_hi + (size_t)(live ? col : 0) * Kp + kg * 8 + (size_t)wave * TPS * 32;
    const uint16_t* bl_base = act_lo + (size_t)(live ? col : 0) * Kp + kg * 8 + (size_t)wave * TPS * 32;
    const v4u zero = (v4u){0u, 0u, 0u, 0u};
    v4u bh[3], bl[3];
#pragma unroll
    for (int j = 0; j < 2 && j < TPS; ++j) {
        bh[j] = live ? *reinterpret_cast<const v4u*>(bh_base + j * 32) : zero;
        bl[j] = live ? *reinterpret_cast<const v4u*>(bl_base + j * 32) : zero;
    }
#pragma unroll
    for (int j = 0; j < TPS; ++j) {
        if (j + 2 < TPS) {
            bh[(j + 2) % 3] = live ? *reinterpret_cast<const v4u*>(bh_base + (j + 2) * 32) : zero;
            bl[(j + 2) % 3] = live ? *reinterpret_cast<const v4u*>(bl_base + (j + 2) * 32) : zero;
        }
        const bf16x8 h = __builtin_bit_cast(bf16x8, bh[j % 3]), l = __builtin_bit_cast(bf16x8, bl[j % 3]);
#pragma unroll
        for (int si = 0; si < NS; ++si) {
            if (si < nstrips) {
                const bf16x8 a = __builtin_bit_cast(bf16x8, w[si * TPS + j]);
                acc[si] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, h, acc[si], 0, 0, 0);
                acc[si] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, l, acc[si], 0, 0, 0);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    }
}

struct RowPos { int seq, r, pos; bool valid; };
__device__ __forceinline__ RowPos row_pos(const SP& p, int c) {
    RowPos o;
    o.seq = c / p.RS;
    o.r = c - o.seq * p.RS;
    const int b = o.seq % p.B;
    const int ke = p.k_eff[b];
    o.valid = o.r <= ke;
    o.pos = o.valid ? p.C + p.n[b] - 1 + o.r : 0;
    return o;
}

// ------------------------------------------------------------------------- GEMV phases

// vals[si][row][col] holds the finished strip; writes it where the next stage expects it.
template <int KIND>
__device__ __forceinline__ void epilogue(const SP& p, int layer, int strip, const float* vals, int lane) {
    const int MR = p.MR, d = p.d;
    if (KIND == K_A) {
        const int o0 = strip * 16, seg = o0 / d, j0 = o0 - seg * d;
        const int hd = d / p.H;
        for (int idx = lane; idx < 8 * MR; idx += 64) {
            const int t = idx & 7, c = idx >> 3;
            float e0 = vals[(2 * t) * 16 + c], e1 = vals[(2 * t + 1) * 16 + c];
            const RowPos rp = row_pos(p, c);
            if (seg < 2) {
                const float2 cs = p.rope[(size_t)rp.pos * (hd / 2) + ((j0 % hd) >> 1) + t];
                const float a = e0 * cs.x - e1 * cs.y, b = e0 * cs.y + e1 * cs.x;
                e0 = a; e1 = b;
            }
            if (seg == 0) {
                st_f32x2(p.Q + (size_t)c * d + j0 + 2 * t, e0, e1);
            } else if (rp.valid) {
                _Float16* dst = (seg == 1 ? p.Kc : p.Vc) +
                                (((size_t)layer * p.Smax + rp.seq) * p.Tmax + rp.pos) * d + j0 + 2 * t;
                const _Float16 h0 = (_Float16)e0, h1 = (_Float16)e1;
                const unsigned pk = (unsigned)__builtin_bit_cast(unsigned short, h0) |
                                    ((unsigned)__builtin_bit_cast(unsigned short, h1) << 16);
                __hip_atomic_store(reinterpret_cast<unsigned*>(dst), pk, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
    } else if (KIND == K_C || KIND == K_E) {
        const float* in = KIND == K_C ? p.X : p.X2;
        float* out = KIND == K_C ? p.X2 : p.X;
        for (int e = lane; e < 16 * MR; e += 64) {
            const int row = e & 15, c = e >> 4;
            const size_t at = (size_t)c * d + strip * 16 + row;
            st_f32(out + at, ld_f32(in + at) + vals[row * 16 + c]);
        }
    } else if (KIND == K_D) {
        for (int e = lane; e < 8 * MR; e += 64) {
            const int i = e & 7, c = e >> 3;
            const float u1 = vals[i * 16 + c], u3 = vals[(8 + i) * 16 + c];
            st_f32(p.Hb + (size_t)c * p.m + strip * 8 + i, u1 / (1.0f + expf(-u1)) * u3);
        }
    } else if (KIND == K_LM) {
        for (int e = lane; e < 16 * MR; e += 64) {
            const int row = e & 15, c = e >> 4;
            p.logit_s[(size_t)c * p.Vs + strip * 16 + row] = vals[row * 16 + c];
        }
    }
}

struct Lds {
    uint16_t* act_hi;
    uint16_t* act_lo;
    float* red;   // [kCW][kMaxStrips][64][4]
    float* vals;  // [kMaxStrips][16][16]
    float* att;   // attention scratch
};

template <int KIND, int TPS, bool NORM, int KREG>
__device__ __forceinline__ void gemv_phase(const SP& p, const Lds& s, Barrier& bar, int layer, int round,
                                           const float* src, int K, const uint16_t* gain) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const bool is_io = wave >= kCW;
    const Job job = load_job(p, KIND, round, layer);
    // The weights do not depend on the previous stage: their loads go out before the barrier is
    // crossed and land while the IO waves synchronise and stage the input.
    v4u w[kTMax];
    if (!is_io) issue_tiles(p, job, TPS, wave, lane, w);
    if (is_io) {
        bar.wait();
        if (job.nstrips) stage_rows<NORM, KREG>(src, K, p.MR, gain, p.eps, wave - kCW, lane, s.act_hi, s.act_lo, p.Kp);
    }
    __syncthreads();
    if (!is_io && job.nstrips) {
        f32x4 acc[kMaxStrips];
#pragma unroll
        for (int i = 0; i < kMaxStrips; ++i) acc[i] = (f32x4){0.f, 0.f, 0.f, 0.f};
        mfma_job<TPS>(w, job.nstrips, wave, lane, p.MR, s.act_hi, s.act_lo, p.Kp, acc);
#pragma unroll
        for (int i = 0; i < kMaxStrips; ++i)
            if (i < job.nstrips) *reinterpret_cast<f32x4*>(s.red + (((size_t)wave * kMaxStrips + i) * 64 + lane) * 4) = acc[i];
    }
    __syncthreads();
    if (wave == kCW) {
#pragma unroll
        for (int i = 0; i < kMaxStrips; ++i) {
            if (i < job.nstrips) {
                // sum the four K quarters; lane holds rows 4*(lane/16)..+3 of column lane%16
                f32x4 v = (f32x4){0.f, 0.f, 0.f, 0.f};
                for (int cw = 0; cw < kCW; ++cw)
                    v += *reinterpret_cast<const f32x4*>(s.red + (((size_t)cw * kMaxStrips + i) * 64 + lane) * 4);
                float* vs = s.vals + (size_t)i * 256;
#pragma unroll
                for (int q = 0; q < 4; ++q) vs[((lane >> 4) * 4 + q) * 16 + (lane & 15)] = v[q];
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): the LDS writes above are visible to the wave
                epilogue<KIND>(p, layer, job.strip[i], vs, lane);
                __builtin_amdgcn_wave_barrier();
            }
        }
        __builtin_amdgcn_s_waitcnt(0);  // results are out before this workgroup arrives
        if (lane == 0) bar.arrive(); else ++bar.id;
    } else {
        ++bar.id;
    }
}

// ------------------------------------------------------------------------- attention

// Stage 1: workgroup (seq, head, chunk) reduces its slice of cache positions for the RS rows
// of its sequence to an un-normalised partial (m, l, o~).  RSMAX bounds the register arrays.
template <int RSMAX>
__device__ __forceinline__ void attn_partial(const SP& p, const Lds& s, Barrier& bar, int layer) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const bool is_io = wave >= kCW;
    const int njobs = p.S * p.H * p.NC;
    const int wg = blockIdx.x;
    const bool have = wg < njobs;
    const int seq = wg / (p.H * p.NC), h = (wg / p.NC) % p.H, ch = wg % p.NC;
    const int d = p.d, RS = p.RS;
    float* qs = s.att;                      // [RS][64] scaled queries
    float* part = s.att + 8 * 64;           // [kCW][RS][66]
    if (is_io) {
        bar.wait();
        if (have && wave == kCW)
            for (int r = 0; r < RS; ++r) qs[r * 64 + lane] = ld_f32(p.Q + (size_t)(seq * RS + r) * d + h * 64 + lane) * 0.125f;
    }
    __syncthreads();
    if (!is_io && have) {
        const int b = seq % p.B, ke = p.k_eff[b];
        const int kv0 = ke >= 0 ? p.C + p.n[b] - 1 : 0;   // cached positions before this step
        const int total = ke >= 0 ? kv0 + ke + 1 : 0;     // positions any row may attend
        const int p0 = (int)((long long)total * ch / p.NC), p1 = (int)((long long)total * (ch + 1) / p.NC);
        const int pg = lane >> 3, dg = lane & 7;
        float acc[RSMAX][8], mx[RSMAX], den[RSMAX];
#pragma unroll
        for (int r = 0; r < RSMAX; ++r) {
            mx[r] = -1e30f; den[r] = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[r][e] = 0.f;
        }
        const size_t base = (((size_t)layer * p.Smax + seq) * p.Tmax) * d + (size_t)h * 64 + dg * 8;
        for (int pos = p0 + wave * 8 + pg; pos < p1; pos += kCW * 8) {
            uint4 kraw, vraw;
            const _Float16* kp = p.Kc + base + (size_t)pos * d;
            const _Float16* vp = p.Vc + base + (size_t)pos * d;
            if (pos >= kv0) {  // written by this launch: device-coherent loads
                u64 a0 = __hip_atomic_load(reinterpret_cast<const u64*>(kp), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                u64 a1 = __hip_atomic_load(reinterpret_cast<const u64*>(kp) + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                u64 b0 = __hip_atomic_load(reinterpret_cast<const u64*>(vp), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                u64 b1 = __hip_atomic_load(reinterpret_cast<const u64*>(vp) + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                kraw = make_uint4((unsigned)a0, (unsigned)(a0 >> 32), (unsigned)a1, (unsigned)(a1 >> 32));
                vraw = make_uint4((unsigned)b0, (unsigned)(b0 >> 32), (unsigned)b1, (unsigned)(b1 >> 32));
            } else {
                kraw = *reinterpret_cast<const uint4*>(kp);
                vraw = *reinterpret_cast<const uint4*>(vp);
            }
            float kf[8], vf[8];
            const unsigned ku[4] = {kraw.x, kraw.y, kraw.z, kraw.w}, vu[4] = {vraw.x, vraw.y, vraw.z, vraw.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                kf[2 * e] = (float)__builtin_bit_cast(_Float16, (unsigned short)(ku[e] & 0xFFFFu));
                kf[2 * e + 1] = (float)__builtin_bit_cast(_Float16, (unsigned short)(ku[e] >> 16));
                vf[2 * e] = (float)__builtin_bit_cast(_Float16, (unsigned short)(vu[e] & 0xFFFFu));
                vf[2 * e + 1] = (float)__builtin_bit_cast(_Float16, (unsigned short)(vu[e] >> 16));
            }
#pragma unroll
            for (int r = 0; r < RSMAX; ++r) {
                if (r < RS) {
                    const float4 qa = *reinterpret_cast<const float4*>(qs + r * 64 + dg * 8);
                    const float4 qb = *reinterpret_cast<const float4*>(qs + r * 64 + dg * 8 + 4);
                    float sc = qa.x * kf[0] + qa.y * kf[1] + qa.z * kf[2] + qa.w * kf[3] + qb.x * kf[4] + qb.y * kf[5] +
                               qb.z * kf[6] + qb.w * kf[7];
                    sc += __shfl_xor(sc, 1, 64);
                    sc += __shfl_xor(sc, 2, 64);
                    sc += __shfl_xor(sc, 4, 64);
                    if (pos <= kv0 + r && r <= ke) {  // causal inside the block of new rows
                        const float mn = fmaxf(mx[r], sc);
                        const float corr = __expf(mx[r] - mn), pw = __expf(sc - mn);
                        den[r] = den[r] * corr + pw;
#pragma unroll
                        for (int e = 0; e < 8; ++e) acc[r][e] = acc[r][e] * corr + pw * vf[e];
                        mx[r] = mn;
                    }
                }
            }
        }
        // merge the 8 position groups of the wave (lanes that share dg), then hand over to LDS
#pragma unroll
        for (int r = 0; r < RSMAX; ++r) {
            if (r < RS) {
                float m2 = mx[r];
                m2 = fmaxf(m2, __shfl_xor(m2, 8, 64));
                m2 = fmaxf(m2, __shfl_xor(m2, 16, 64));
                m2 = fmaxf(m2, __shfl_xor(m2, 32, 64));
                const float f = __expf(mx[r] - m2);
                float dn = den[r] * f;
                dn += __shfl_xor(dn, 8, 64); dn += __shfl_xor(dn, 16, 64); dn += __shfl_xor(dn, 32, 64);
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    float a = acc[r][e] * f;
                    a += __shfl_xor(a, 8, 64); a += __shfl_xor(a, 16, 64); a += __shfl_xor(a, 32, 64);
                    if (pg == 0) part[((size_t)wave * RS + r) * 66 + dg * 8 + e] = a;
                }
                if (lane == 0) { part[((size_t)wave * RS + r) * 66 + 64] = m2; part[((size_t)wave * RS + r) * 66 + 65] = dn; }
            }
        }
    }
    __syncthreads();
    if (wave == kCW) {
        if (have) {
            float* out = p.P + (size_t)wg * RS * 66;
            for (int r = 0; r < RS; ++r) {
                float m2 = -1e30f;
                for (int cw = 0; cw < kCW; ++cw) m2 = fmaxf(m2, part[((size_t)cw * RS + r) * 66 + 64]);
                float dn = 0.f, o = 0.f;
                for (int cw = 0; cw < kCW; ++cw) {
                    const float f = __expf(part[((size_t)cw * RS + r) * 66 + 64] - m2);
                    dn += part[((size_t)cw * RS + r) * 66 + 65] * f;
                    o += part[((size_t)cw * RS + r) * 66 + lane] * f;
                }
                st_f32(out + r * 66 + lane, o);
                if (lane == 0) st_f32x2(out + r * 66 + 64, m2, dn);
            }
        }
        __builtin_amdgcn_s_waitcnt(0);
        if (lane == 0) bar.arrive(); else ++bar.id;
    } else {
        ++bar.id;
    }
}

// Stage 2: workgroup (seq, head) merges the NC chunk partials into the attention output.
__device__ __forceinline__ void attn_merge(const SP& p, Barrier& bar) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const bool is_io = wave >= kCW;
    if (is_io) bar.wait();
    __syncthreads();
    if (wave == kCW) {
        const int wg = blockIdx.x;
        if (wg < p.S * p.H) {
            const int seq = wg / p.H, h = wg % p.H;
            for (int r = 0; r < p.RS; ++r) {
                float m2 = -1e30f;
                const float* src = p.P + ((size_t)wg * p.NC) * p.RS * 66 + (size_t)r * 66;
                for (int c = 0; c < p.NC; ++c) m2 = fmaxf(m2, ld_f32(src + (size_t)c * p.RS * 66 + 64));
                float dn = 0.f, o = 0.f;
                for (int c = 0; c < p.NC; ++c) {
                    const float f = __expf(ld_f32(src + (size_t)c * p.RS * 66 + 64) - m2);
                    dn += ld_f32(src + (size_t)c * p.RS * 66 + 65) * f;
                    o += ld_f32(src + (size_t)c * p.RS * 66 + lane) * f;
                }
                st_f32(p.O + (size_t)(seq * p.RS + r) * p.d + h * 64 + lane, dn > 0.f ? o / dn : 0.f);
            }
        }
        __builtin_amdgcn_s_waitcnt(0);
        if (lane == 0) bar.arrive(); else ++bar.id;
    } else {
        ++bar.id;
    }
    __syncthreads();
}

// ------------------------------------------------------------------------- the kernel

template <int TPS_D, int TPS_M, int KREG_D, int KREG_M, int RSMAX>
__global__ __launch_bounds__(kThreads, 1) void verify_stream_kernel(SP p) {
    extern __shared__ uint4 smem_raw[];
    Lds s;
    s.act_hi = reinterpret_cast<uint16_t*>(smem_raw);
    s.act_lo = s.act_hi + (size_t)p.MR * p.Kp;
    s.red = reinterpret_cast<float*>(s.act_lo + (size_t)p.MR * p.Kp);
    s.vals = s.red + kCW * kMaxStrips * 64 * 4;
    s.att = s.vals + kMaxStrips * 256;
    Barrier bar;
    bar.mem = p.bar; bar.err = p.err; bar.id = p.epoch0; bar.first = p.epoch0; bar.dead = false;
    for (int l = 0; l < p.L; ++l) {
        const uint16_t* g1 = p.blob + (p.g1_off + (u64)l * p.layer_bytes) / 2;
        const uint16_t* g2 = p.blob + (p.g2_off + (u64)l * p.layer_bytes) / 2;
        gemv_phase<K_A, TPS_D, true, KREG_D>(p, s, bar, l, 0, p.X, p.d, g1);
        attn_partial<RSMAX>(p, s, bar, l);
        attn_merge(p, bar);
        gemv_phase<K_C, TPS_D, false, KREG_D>(p, s, bar, l, 0, p.O, p.d, nullptr);
        gemv_phase<K_D, TPS_D, true, KREG_D>(p, s, bar, l, 0, p.X2, p.d, g2);
        gemv_phase<K_E, TPS_M, false, KREG_M>(p, s, bar, l, 0, p.Hb, p.m, nullptr);
    }
    const uint16_t* gf = p.blob + p.gf_off / 2;
    for (int r = 0; r < p.rounds[K_LM]; ++r)
        gemv_phase<K_LM, TPS_D, true, KREG_D>(p, s, bar, p.L - 1, r, p.X, p.d, gf);
}

// Copies one matrix into the tile order of its kind: tile T of the packed stream is
// (strip, k-tile) = desc[T]; lane l holds row l%16, columns 8*(l/16)..+7 of that tile.
__global__ void repack_kernel(const uint16_t* W, int K, int kind, int m, int row0, const uint32_t* desc, uint4* out) {
    const size_t tile = blockIdx.x;
    const int lane = threadIdx.x;
    const uint32_t dsc = desc[tile];
    const int strip = dsc >> 12, kt = dsc & 4095, r = lane & 15;
    const size_t row = kind == K_D ? (size_t)((r < 8 ? 0 : m) + strip * 8 + (r & 7)) : (size_t)(row0 + strip * 16 + r);
    out[tile * 64 + lane] = *reinterpret_cast<const uint4*>(W + row * K + kt * 32 + (lane >> 4) * 8);
}

// ------------------------------------------------------------------------- host: plan

struct KindPlan {
    int nstrips, KT, TPS, maxS, rounds;
    size_t tiles;        // tiles of one instance of this kind
    size_t tab_index;    // int32 index of the job table
    size_t desc_index;   // uint32 index of the tile descriptors
};

}  // namespace

struct StreamPlan {
    bool ok;
    KindPlan kind[K_NKIND];
    size_t layer_tiles, kind_base[4], lm_base, wd_base, total_tiles;
    std::vector<int32_t> tab;
    std::vector<uint32_t> desc;
    std::vector<uint32_t> hasmask;
    unsigned epoch;
    size_t lds_bytes_per_row;
};

namespace {

bool shape_ok(const hawk_ctx* c) {
    if (c->cfg.dtype != HAWK_BF16) return false;
    if (c->hd != 64) return false;
    if (c->d % 128 || c->m % 128 || c->Vs % 16 || (3 * c->d) % 128) return false;
    if (c->d / 128 > kTMax || c->m / 128 > kTMax || 3 * c->d / 128 > kTMax) return false;
    if (!((c->d == 1280 && c->m == 3456) || (c->d == 768 && c->m == 2048))) return false;  // instantiated tilings
    if (c->Vs / 16 > 65535 || (2 * c->m) / 16 > 65535) return false;
    return true;
}

// Spreads the strips of the layer kinds over the workgroups so that every workgroup streams
// about the same number of tiles per layer: heaviest strips first, each to the least loaded
// workgroup that still has room in that kind.
void build_plan(const hawk_ctx* c, StreamPlan* P) {
    P->ok = shape_ok(c);
    if (!P->ok) return;
    const int d = c->d, m = c->m;
    const int nstrips[K_NKIND] = {3 * d / 16, d / 16, 2 * m / 16, d / 16, c->Vs / 16, d / 16};
    const int KT[K_NKIND] = {d / 32, d / 32, d / 32, m / 32, d / 32, 3 * d / 32};
    for (int k = 0; k < K_NKIND; ++k) {
        KindPlan& kp = P->kind[k];
        kp.nstrips = nstrips[k]; kp.KT = KT[k]; kp.TPS = KT[k] / 4;
        kp.maxS = std::min(kMaxStrips, kTMax / kp.TPS);
        kp.tiles = (size_t)nstrips[k] * KT[k];
        kp.rounds = k <= K_E ? 1 : (nstrips[k] + kNWG * kp.maxS - 1) / (kNWG * kp.maxS);
        if (k <= K_E && nstrips[k] > kNWG * kp.maxS) { P->ok = false; return; }
    }
    std::vector<std::vector<int>> assign[K_NKIND];  // [kind][round][wg] -> strips
    for (int k = 0; k < K_NKIND; ++k) assign[k].assign((size_t)P->kind[k].rounds * kNWG, {});
    std::vector<long> load(kNWG, 0);
    int order[4] = {K_A, K_C, K_D, K_E};
    std::sort(order, order + 4, [&](int a, int b) { return P->kind[a].TPS > P->kind[b].TPS; });
    for (int oi = 0; oi < 4; ++oi) {
        const int k = order[oi];
        for (int s = 0; s < nstrips[k]; ++s) {
            int best = -1;
            for (int g = 0; g < kNWG; ++g)
                if ((int)assign[k][g].size() < P->kind[k].maxS && (best < 0 || load[g] < load[best])) best = g;
            assign[k][best].push_back(s);
            load[best] += P->kind[k].TPS;
        }
    }
    for (int k = K_LM; k <= K_WD; ++k) {  // output projection and draft projection: round robin
        int s = 0;
        for (int r = 0; r < P->kind[k].rounds; ++r) {
            const int left = nstrips[k] - s, rounds_left = P->kind[k].rounds - r;
            const int per_round = (left + rounds_left - 1) / rounds_left;
            for (int i = 0; i < per_round; ++i, ++s) assign[k][(size_t)r * kNWG + i % kNWG].push_back(s);
        }
    }
    P->tab.clear(); P->desc.clear();
    P->hasmask.assign(kNWG, 0);
    for (int k = 0; k < K_NKIND; ++k) {
        KindPlan& kp = P->kind[k];
        kp.tab_index = P->tab.size();
        kp.desc_index = P->desc.size();
        uint32_t tile = 0;
        for (int r = 0; r < kp.rounds; ++r)
            for (int g = 0; g < kNWG; ++g) {
                const std::vector<int>& st = assign[k][(size_t)r * kNWG + g];
                const int ns = (int)st.size();
                int s3[3] = {0xFFFF, 0xFFFF, 0xFFFF};
                for (int i = 0; i < ns; ++i) s3[i] = st[i];
                P->tab.push_back((int32_t)tile);
                P->tab.push_back(ns);
                P->tab.push_back((int32_t)((unsigned)s3[0] | ((unsigned)s3[1] << 16)));
                P->tab.push_back(s3[2]);
                if (ns) P->hasmask[g] |= k <= K_E ? (1u << k) : (k == K_LM ? (1u << (8 + r)) : 0u);
                for (int wv = 0; wv < kCW; ++wv)
                    for (int t = 0; t < ns * kp.TPS; ++t) {
                        P->desc.push_back(((uint32_t)st[t / kp.TPS] << 12) | (uint32_t)(wv * kp.TPS + t % kp.TPS));
                        ++tile;
                    }
            }
    }
    size_t off = 0;
    for (int k = 0; k <= K_E; ++k) { P->kind_base[k] = off; off += P->kind[k].tiles; }
    P->layer_tiles = off;
    P->lm_base = (size_t)c->L * P->layer_tiles;
    P->wd_base = P->lm_base + P->kind[K_LM].tiles;
    P->total_tiles = P->wd_base + P->kind[K_WD].tiles;
    // every tile of every kind has been placed exactly once
    size_t placed = 0;
    for (int k = 0; k < K_NKIND; ++k) placed += P->kind[k].tiles;
    if (P->desc.size() != placed) P->ok = false;
}

size_t up256(size_t x) { return (x + 255) & ~(size_t)255; }

}  // namespace

// Bytes the streaming path adds to the workspace (0 if the shape is not supported), and the
// offsets of its regions relative to `base`.
size_t stream_workspace(const hawk_ctx* c, size_t base, StreamOffsets* o) {
    memset(o, 0, sizeof *o);
    if (!shape_ok(c)) return 0;
    const size_t d = c->d, m = c->m, L = c->L;
    const size_t tiles = L * (4 * d * d + 3 * d * m) / 512 + (size_t)c->Vs * d / 512 + 3 * d * d / 512;
    size_t p = base;
    auto take = [&](size_t bytes) { size_t at = p; p = up256(p + bytes); return at; };
    o->wpack = take(tiles * 1024);
    o->tab = take((size_t)(K_NKIND + (size_t)c->Vs / 16 / kNWG + 2) * kNWG * 16);
    o->desc = take(((4 * d * d + 3 * d * m) / 512 + (size_t)c->Vs * d / 512 + 3 * d * d / 512 + 64) * 4);
    o->hasmask = take(kNWG * 4);
    o->x2 = take(16 * d * 4); o->q = take(16 * d * 4); o->o = take(16 * d * 4); o->h = take(16 * m * 4);
    o->p = take((size_t)kNWG * 8 * 66 * 4);
    o->bar = take((size_t)(kGroups + 1 + kReplicas) * 4096);
    o->err = take(256);
    o->rope = take((size_t)c->Tmax * (c->hd / 2) * 8);
    return p - base;
}

StreamPlan* stream_create(hawk_ctx* c) {
    StreamPlan* P = new StreamPlan();
    build_plan(c, P);
    P->epoch = 0;
    if (!P->ok) return P;
    const StreamOffsets& o = c->soff;
    // tables, rotary table, zeroed barrier memory
    (void)hipMemcpy(c->ws + o.tab, P->tab.data(), P->tab.size() * 4, hipMemcpyHostToDevice);
    (void)hipMemcpy(c->ws + o.desc, P->desc.data(), P->desc.size() * 4, hipMemcpyHostToDevice);
    (void)hipMemcpy(c->ws + o.hasmask, P->hasmask.data(), P->hasmask.size() * 4, hipMemcpyHostToDevice);
    (void)hipMemset(c->ws + o.bar, 0, (size_t)(kGroups + 1 + kReplicas) * 4096);
    (void)hipMemset(c->ws + o.err, 0, 256);
    std::vector<float> rope((size_t)c->Tmax * (c->hd / 2) * 2);
    for (int pos = 0; pos < c->Tmax; ++pos)
        for (int j = 0; j < c->hd / 2; ++j) {
            const double ang = (double)pos * pow((double)c->cfg.rope_theta, -2.0 * j / (double)c->hd);
            rope[((size_t)pos * (c->hd / 2) + j) * 2] = (float)cos(ang);
            rope[((size_t)pos * (c->hd / 2) + j) * 2 + 1] = (float)sin(ang);
        }
    (void)hipMemcpy(c->ws + o.rope, rope.data(), rope.size() * 4, hipMemcpyHostToDevice);
    return P;
}

void stream_destroy(StreamPlan* P) { delete P; }

// Host-only summary of the streaming plan of a configuration (no device access).
// out[0] supported, [1] tiles per layer, [2] tiles in total, [3]/[4] fewest / most tiles any
// workgroup streams per layer, [5] output-projection rounds, [6] 1 if every table entry and
// tile descriptor is inside its matrix, [7] workgroups.
void stream_plan_info(const hawk_ctx* c, int64_t* out) {
    StreamPlan P;
    build_plan(c, &P);
    for (int i = 0; i < 8; ++i) out[i] = 0;
    out[7] = kNWG;
    if (!P.ok) return;
    out[0] = 1;
    out[1] = (int64_t)P.layer_tiles;
    out[2] = (int64_t)P.total_tiles;
    std::vector<long> load(kNWG, 0);
    bool sane = true;
    for (int k = 0; k < K_NKIND; ++k) {
        const KindPlan& kp = P.kind[k];
        std::vector<int> seen((size_t)kp.nstrips * kp.KT, 0);
        size_t tile = 0;
        for (int r = 0; r < kp.rounds; ++r)
            for (int g = 0; g < kNWG; ++g) {
                const int32_t* e = &P.tab[kp.tab_index + ((size_t)r * kNWG + g) * 4];
                const int ns = e[1];
                sane = sane && ns >= 0 && ns <= kp.maxS && (size_t)e[0] == tile && ns * kp.TPS <= kTMax;
                if (k <= K_E) load[g] += (long)ns * kp.TPS * kCW;
                for (int t = 0; t < ns * kp.TPS * kCW; ++t, ++tile) {
                    const uint32_t dsc = P.desc[kp.desc_index + tile];
                    const int strip = (int)(dsc >> 12), kt = (int)(dsc & 4095);
                    if (strip >= kp.nstrips || kt >= kp.KT) { sane = false; continue; }
                    seen[(size_t)strip * kp.KT + kt] += 1;
                }
            }
        sane = sane && tile == kp.tiles;
        for (int v : seen) sane = sane && v == 1;
    }
    out[3] = *std::min_element(load.begin(), load.end());
    out[4] = *std::max_element(load.begin(), load.end());
    out[5] = P.kind[K_LM].rounds;
    out[6] = sane ? 1 : 0;
}

bool stream_ok(const hawk_ctx* c, int k) {
    if (!c->plan || !c->plan->ok || c->path != 1) return false;
    const int MR = c->S * (k + 1);
    if (MR > 16 || k + 1 > 6) return false;
    if (c->S * c->H > kNWG) return false;
    const size_t lds = (size_t)MR * (std::max(c->d, c->m) + 8) * 4 + (kCW * kMaxStrips * 256 + kMaxStrips * 256) * 4 +
                       (8 * 64 + kCW * 8 * 66) * 4;
    return lds <= 150 * 1024;
}

// Re-tiles every matrix of the loaded blob into the streaming order (after hawk_load).
int stream_repack(hawk_ctx* c) {
    StreamPlan* P = c->plan;
    if (!P || !P->ok) return 0;
    const uint16_t* blob = wsp<uint16_t>(c, c->off.blob);
    uint4* wp = wsp<uint4>(c, c->soff.wpack);
    const uint32_t* desc = wsp<uint32_t>(c, c->soff.desc);
    auto run = [&](size_t blob_off, int K, int kind, size_t tile_base, int row0) {
        const KindPlan& kp = P->kind[kind];
        repack_kernel<<<(unsigned)kp.tiles, 64, 0, c->stream>>>(blob + blob_off / 2, K, kind, c->m, row0,
                                                              desc + kp.desc_index, wp + tile_base * 64);
    };
    for (int l = 0; l < c->L; ++l) {
        const size_t lb = (size_t)l * P->layer_tiles;
        run(c->w.Wqkv[l], c->d, K_A, lb + P->kind_base[K_A], 0);
        run(c->w.Wo[l], c->d, K_C, lb + P->kind_base[K_C], 0);
        run(c->w.W13[l], c->d, K_D, lb + P->kind_base[K_D], 0);
        run(c->w.W2[l], c->m, K_E, lb + P->kind_base[K_E], 0);
    }
    run(c->w.W_out, c->d, K_LM, P->lm_base, c->cfg.samp_lo);
    run(c->w.W_d, 3 * c->d, K_WD, P->wd_base, 0);
    if (hipGetLastError() != hipSuccess) return -1;
    return hipStreamSynchronize(c->stream) == hipSuccess ? 0 : -1;
}

// Enqueues the target pass over the step rows; X (c->off.x) must hold the embedded rows.
// Returns 0, or -1 if the launch failed.
int launch_verify_stream(hawk_ctx* c, int k) {
    StreamPlan* P = c->plan;
    SP p;
    memset(&p, 0, sizeof p);
    const StreamOffsets& o = c->soff;
    p.wpack = wsp<uint4>(c, o.wpack);
    p.layer_tiles = P->layer_tiles;
    for (int i = 0; i < 4; ++i) p.kind_base[i] = P->kind_base[i];
    p.lm_base = P->lm_base; p.wd_base = P->wd_base;
    for (int i = 0; i < K_NKIND; ++i) {
        p.tab[i] = wsp<int32_t>(c, o.tab) + P->kind[i].tab_index;
        p.rounds[i] = P->kind[i].rounds;
    }
    p.hasmask = wsp<uint32_t>(c, o.hasmask);
    p.blob = wsp<uint16_t>(c, c->off.blob);
    p.g1_off = c->w.g1[0]; p.g2_off = c->w.g2[0];
    p.layer_bytes = c->L > 1 ? c->w.g1[1] - c->w.g1[0] : 0;
    p.gf_off = c->w.g_f;
    p.rope = wsp<float2>(c, o.rope);
    p.Kc = wsp<_Float16>(c, c->off.kc); p.Vc = wsp<_Float16>(c, c->off.vc);
    p.X = wsp<float>(c, c->off.x); p.X2 = wsp<float>(c, o.x2); p.Q = wsp<float>(c, o.q); p.P = wsp<float>(c, o.p);
    p.O = wsp<float>(c, o.o); p.Hb = wsp<float>(c, o.h); p.logit_s = wsp<float>(c, c->off.logit_s);
    p.bar = wsp<unsigned>(c, o.bar); p.err = wsp<unsigned>(c, o.err);
    p.n = wsp<int32_t>(c, c->off.n); p.k_eff = wsp<int32_t>(c, c->off.k_eff);
    p.epoch0 = P->epoch;
    p.L = c->L; p.d = c->d; p.H = c->H; p.m = c->m; p.Vs = c->Vs; p.S = c->S; p.B = c->B; p.C = c->C;
    p.RS = k + 1; p.MR = c->S * (k + 1);
    p.NC = std::max(1, kNWG / (c->S * c->H));
    p.Smax = c->Smax; p.Tmax = c->Tmax; p.Kp = std::max(c->d, c->m) + 8;
    p.eps = c->cfg.rms_eps;
    const size_t lds = (size_t)p.MR * p.Kp * 4 + (kCW * kMaxStrips * 256 + kMaxStrips * 256) * 4 + (8 * 64 + kCW * 8 * 66) * 4;
    const void* kern = c->d == 1280 ? reinterpret_cast<const void*>(verify_stream_kernel<10, 27, 10, 27, 6>)
                                    : reinterpret_cast<const void*>(verify_stream_kernel<6, 16, 6, 16, 6>);
    if (hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess) return -1;
    void* args[] = {&p};
    if (hipLaunchCooperativeKernel(kern, dim3(kNWG), dim3(kThreads), args, lds, c->stream) != hipSuccess) return -1;
    P->epoch += 6u * (unsigned)c->L + (unsigned)P->kind[K_LM].rounds;
    return 0;
}

// 1 if a barrier of the streaming kernels ever timed out (the result of that step is invalid).
int stream_error(hawk_ctx* c) {
    if (!c->plan || !c->plan->ok) return 0;
    unsigned e = 0;
    if (hipMemcpyAsync(&e, c->ws + c->soff.err, 4, hipMemcpyDeviceToHost, c->stream) != hipSuccess) return 1;
    if (hipStreamSynchronize(c->stream) != hipSuccess) return 1;
    return e != 0;
}

}  // namespace hawk
