// Weight-streaming verify pass: the whole target pass over the k+1 rows of every sequence
// (all layers + output projection) as ONE persistent kernel of 256 workgroups, one per CU.
//
// Why this shape (MI355X, measured): at batch 1 a layer of the XL model is 40 MB, i.e. ~5 us
// of HBM time, but it has five dependent stages; a kernel boundary costs ~6 us for an 8 MB
// kernel and a store -> remote load round trip ~1.5 us, so the stages live in one kernel, the
// weights of stage p+1 are in flight while stage p synchronises, and everything on the
// dependent chain of a stage is kept as short as possible:
//   - every matrix is pre-packed into 16x32 bf16 tiles laid out exactly as the A operand of
//     v_mfma_f32_16x16x32_bf16 (16 bytes per lane), in the order each wave consumes them;
//   - a workgroup owns whole 16-row output strips; its four compute waves split K four ways,
//     stream their tiles straight from HBM into VGPRs (no LDS staging of weights) and issue
//     the loads of their NEXT job right after the MFMAs of the current one;
//   - the k+1 activation rows are the B operand (columns 0..MR-1 of 16), kept as a bf16
//     hi + lo pair (two MFMAs per tile: fp32-accurate activations at no HBM cost).  The
//     PRODUCER of a vector writes it already split (and multiplied by the gain of the norm
//     that follows, with per-strip sums of squares beside it), so a consumer only copies
//     16-byte chunks into LDS and applies the row's 1/rms to its accumulators;
//   - the residual stream of a 16-column strip never leaves the workgroup that owns the strip
//     in both the Wo and the W2 stage (four registers per lane of one wave);
//   - four IO waves per workgroup do everything latency-bound: cross the barrier, copy the
//     stage input, reduce the K quarters and write the strips' results (one wave per strip);
//     compute waves never wait on anything but their own weights;
//   - a grid barrier = arrival counters in 16 groups + top counter + replicated release word
//     (1.5 us measured; flat counters or all-to-all flags are 2-3x slower on 8 XCDs).
// Attention reads the fp16 KV cache with (sequence, head, row group, chunk) jobs; with one
// chunk per head the job emits the finished, split output row itself.
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
constexpr int kNIO = 4;                         // IO waves per workgroup
constexpr int kThreads = (kCW + kNIO) * 64;
constexpr int kIOThreads = kNIO * 64;
constexpr int kTMax = 27;                       // tiles (1 KB each) a wave holds for one job
constexpr int kMaxStrips = 3;                   // strips of one job (one IO wave finishes each)
constexpr int kGroups = 8, kReplicas = 8;       // barrier fan-in (one group per XCD) / release fan-out
constexpr unsigned kSpinLimit = 1u << 21;
constexpr int kRing = 3;                        // exchange arenas used round robin by successive launches
constexpr int kPS = 68;                         // floats per attention partial row: 64 outputs, max, sum, pad
constexpr int kNIT = 6;                         // iterations (of kCW*8 cache positions) per KV register buffer
constexpr int kNCMax = 4;                       // chunks per (sequence, head)
constexpr int kXcd = 8, kPerXcd = kNWG / kXcd;  // workgroup i is dispatched to XCD i % 8

// ------------------------------------------------------------------------- kernel parameters

struct SP {
    const uint4* wpack;
    u64 layer_tiles, kind_base[4], lm_base, wd_base;
    const int32_t* tab[K_NKIND];
    int32_t rounds[K_NKIND];
    const uint16_t* blob;
    u64 g1_off, g2_off, layer_bytes, gf_off;
    const float2* rope;
    _Float16* Kc;
    _Float16* Vc;
    float* X;        // embedded rows in, final hidden rows out ([MR][d] fp32)
    float* arena;    // exchange slots of this launch: slot l = arena + l * slot_floats, l = 0..L
    // offsets (in floats) of the regions of a slot: split planes are uint16 [16][K + 8]
    u64 slot_floats, o_xh, o_xl, o_ssx, o_q, o_oh, o_ol, o_x2h, o_x2l, o_ss2, o_hh, o_hl, o_p, o_ep;
    float* logit_s;
    u64* dbg;        // optional per-phase timestamps of the first IO wave of workgroups 0 and 128 (null: off)
    unsigned* bar;
    unsigned* err;
    const int32_t* n;
    const int32_t* k_eff;
    unsigned epoch0;
    int32_t L, d, H, m, Vs, S, B, C, RS, MR, NC, NRG, RPJ, Smax, Tmax, Kpd, Kpm, KpE, esplit, act_bytes;
    float eps;
    // draft head kernel only
    const float* prev;      // [S][d]: hidden state the head continues from
    float* gout;            // [S][d]: the head's output (next micro-step's prev)
    float* dpart;           // [3][16][d]: partial products of the three column blocks of W_d
    const int32_t* grid;
    const int32_t* draft;
    u64 E_off;
    int32_t step_i, N, IW, kstride;
    // tree rows only (see RowMap): depth and ancestor mask of the tree's nodes
    const int32_t* tdepth;
    const u64* tanc;
};

// ------------------------------------------------------------------------- device helpers

// Exchange data is written once per launch, with stores that go through to memory, into a slot
// that no cache has seen in this launch; after the barrier ordinary cached loads return it and
// the 32 workgroups of an XCD share one L2 fill.
__device__ __forceinline__ void st_u32(void* p, unsigned v) {
    __hip_atomic_store(reinterpret_cast<unsigned*>(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_u64(void* p, unsigned lo, unsigned hi) {
    __hip_atomic_store(reinterpret_cast<u64*>(p), (u64)lo | ((u64)hi << 32), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_f32(float* p, float v) { st_u32(p, __float_as_uint(v)); }
__device__ __forceinline__ void st_f32x2(float* p, float a, float b) { st_u64(p, __float_as_uint(a), __float_as_uint(b)); }
__device__ __forceinline__ void st_f32x4(float* p, f32x4 v) {
    st_f32x2(p, v[0], v[1]);
    st_f32x2(p + 2, v[2], v[3]);
}
__device__ __forceinline__ void compiler_fence() { __atomic_signal_fence(__ATOMIC_SEQ_CST); }

// Cross-row lane exchanges in the VALU (gfx950 lane swaps; a shuffle would go through the LDS
// crossbar).  swap16(v, v) returns {rows 0,0,2,2 | rows 1,1,3,3} of v, swap32(v, v) returns
// {lower half twice | upper half twice}: their sum is v[l] + v[l ^ 16] (resp. v[l ^ 32]) in every
// lane, and a select by the lane's own row / half gives the partner's value.
__device__ __forceinline__ float sum_xor16(float v) {
    const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
__device__ __forceinline__ float sum_xor32(float v) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
__device__ __forceinline__ float lane_xor16(float v) {
    const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return __uint_as_float((threadIdx.x & 16u) ? r[0] : r[1]);
}
__device__ __forceinline__ float lane_xor32(float v) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return __uint_as_float((threadIdx.x & 32u) ? r[0] : r[1]);
}
__device__ __forceinline__ float lane_xor8(float v) {   // row_ror:8 - the other half of the 16-lane row
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x128, 0xF, 0xF, true));
}
__device__ __forceinline__ float* slot(const SP& p, int l) { return p.arena + (u64)l * p.slot_floats; }
__device__ __forceinline__ uint16_t* plane(const SP& p, int l, u64 off) {
    return reinterpret_cast<uint16_t*>(slot(p, l) + off);
}

__device__ __forceinline__ unsigned bf16_rne(float f) {
    unsigned u = __float_as_uint(f);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}
__device__ __forceinline__ float bf16_f32(unsigned b) { return __uint_as_float(b << 16); }

// Writes four consecutive elements of a split vector: bf16 hi and lo halves, 8 bytes each.
__device__ __forceinline__ void st_split4(uint16_t* hi, uint16_t* lo, f32x4 v) {
    const unsigned h0 = bf16_rne(v[0]), h1 = bf16_rne(v[1]), h2 = bf16_rne(v[2]), h3 = bf16_rne(v[3]);
    const unsigned l0 = bf16_rne(v[0] - bf16_f32(h0)), l1 = bf16_rne(v[1] - bf16_f32(h1));
    const unsigned l2 = bf16_rne(v[2] - bf16_f32(h2)), l3 = bf16_rne(v[3] - bf16_f32(h3));
    st_u64(hi, h0 | (h1 << 16), h2 | (h3 << 16));
    st_u64(lo, l0 | (l1 << 16), l2 | (l3 << 16));
}
__device__ __forceinline__ void put_split(float4 v, uint16_t* hi, uint16_t* lo) {  // LDS destination
    const unsigned h0 = bf16_rne(v.x), h1 = bf16_rne(v.y), h2 = bf16_rne(v.z), h3 = bf16_rne(v.w);
    const unsigned l0 = bf16_rne(v.x - bf16_f32(h0)), l1 = bf16_rne(v.y - bf16_f32(h1));
    const unsigned l2 = bf16_rne(v.z - bf16_f32(h2)), l3 = bf16_rne(v.w - bf16_f32(h3));
    *reinterpret_cast<uint2*>(hi) = make_uint2(h0 | (h1 << 16), h2 | (h3 << 16));
    *reinterpret_cast<uint2*>(lo) = make_uint2(l0 | (l1 << 16), l2 | (l3 << 16));
}

// Grid barrier.  Counters only ever grow (epochs continue across launches), so nothing is
// reset between kernels.  Waits are bounded: a workgroup that gives up raises *err and stops
// waiting for the rest of the kernel, so that every wave always terminates.
struct Barrier {
    unsigned* mem;
    unsigned* err;
    unsigned id;       // barriers completed so far (global count)
    unsigned first;    // id at kernel start
    unsigned joins;    // io_join calls so far (IO waves)
    bool dead;
    // Arrival in two halves, so that the workgroup can be told that the arrival is on its way
    // (and may queue loads behind it) before the counter's old value has come back.
    __device__ unsigned arrive_issue() {  // one lane of one wave per workgroup
        const unsigned g = blockIdx.x % kGroups;
        return __hip_atomic_fetch_add(mem + (size_t)g * 1024, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __device__ void arrive_finish(unsigned prev) {
        ++id;
        const unsigned per = gridDim.x / kGroups;
        if (prev + 1 == id * per) {  // last of its group: publish the group's word in every replica line
            const unsigned g = blockIdx.x % kGroups;
            for (int r = 0; r < kReplicas; ++r)
                __hip_atomic_store(mem + (size_t)(kGroups + 1 + r) * 1024 + g, id, __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    __device__ void wait() {  // whole wave; returns when barrier `id` has been released
        if (id == first || dead) return;
        // the 16 groups' words of one replica sit in one 64-byte line: lanes 0..15 read one each
        const unsigned l = threadIdx.x & 63u;
        const unsigned* rel = mem + (size_t)(kGroups + 1 + blockIdx.x % kReplicas) * 1024 + (l < (unsigned)kGroups ? l : 0u);
        for (unsigned spins = 0; spins < kSpinLimit; ++spins) {  // one round trip per spin
            unsigned v = __hip_atomic_load(rel, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (__all((int)(v - id) >= 0)) { compiler_fence(); return; }
            if ((spins & 255u) == 255u && __hip_atomic_load(err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u) break;
        }
        dead = true;
        __hip_atomic_store(err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
};

// Timestamp slot `what` (0..7) of phase `phase` (constant 100 MHz clock).
__device__ __forceinline__ void stamp(const SP& p, unsigned phase, int what) {
    if (p.dbg && (threadIdx.x & 63) == 0 && (threadIdx.x >> 6) == kCW && (blockIdx.x & 127) == 0)
        p.dbg[((size_t)(blockIdx.x >> 7) * 4096 + phase) * 8 + what] = __builtin_amdgcn_s_memrealtime();
}

// Same for the first compute wave (second half of the trace buffer).
__device__ __forceinline__ void stamp_c(const SP& p, unsigned phase, int what) {
    if (p.dbg && threadIdx.x == 0 && (blockIdx.x & 127) == 0)
        p.dbg[((size_t)(2 + (blockIdx.x >> 7)) * 4096 + phase) * 8 + what] = __builtin_amdgcn_s_memrealtime();
}

// Every workgroup's arrival (what = 0) and release-seen (what = 1) time of a stage, behind the
// per-wave traces: [what][stage < 256][workgroup].
constexpr size_t kDbgAll = (size_t)4 * 4096 * 8;
__device__ __forceinline__ void stamp_all(const SP& p, unsigned phase, int what) {
    if (p.dbg && phase < 256u && (threadIdx.x & 63) == 0 && (threadIdx.x >> 6) == kCW)
        p.dbg[kDbgAll + ((size_t)what * 256 + phase) * kNWG + blockIdx.x] = __builtin_amdgcn_s_memrealtime();
}

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

// Issues the 16-byte loads of one wave's tiles of a job (nothing is waited for here).  Every
// slot is redefined - zero for a strip the job does not have - so no value outlives its job
// and the MFMA loop needs no branches.
template <int TPS, int NS>
__device__ __forceinline__ void issue_tiles(const SP& p, const Job& j, int wave, int lane, v4u (&w)[NS * TPS]) {
    const int nt = j.nstrips * TPS;
    const v4u* src = reinterpret_cast<const v4u*>(p.wpack + (j.tile0 + (u64)wave * nt) * 64 + lane);
#pragma unroll
    for (int si = 0; si < NS; ++si) {
        if (si < j.nstrips) {
#pragma unroll
            for (int t = 0; t < TPS; ++t) w[si * TPS + t] = __builtin_nontemporal_load(src + (size_t)(si * TPS + t) * 64);
        } else {
#pragma unroll
            for (int t = 0; t < TPS; ++t) w[si * TPS + t] = (v4u){0u, 0u, 0u, 0u};
        }
    }
}

// Copies the split planes of a stage input ([MR][Kp] bf16 each, contiguous) into LDS, BATCH
// 16-byte chunks per IO thread in flight; t = 0..kIOThreads-1.
template <int BATCH>
__device__ __forceinline__ void stage_copy(const uint16_t* hi, const uint16_t* lo, int MR, int Kp, uint16_t* act_hi,
                                           uint16_t* act_lo, int t) {
    const int per_plane = MR * Kp / 8, total = 2 * per_plane;
    for (int base = 0; base < total; base += kIOThreads * BATCH) {
        v4u v[BATCH];
#pragma unroll
        for (int i = 0; i < BATCH; ++i) {
            const int q = base + i * kIOThreads + t;
            const bool second = q >= per_plane;
            const v4u* src = reinterpret_cast<const v4u*>(second ? lo : hi) + (second ? q - per_plane : q);
            v[i] = q < total ? *src : (v4u){0u, 0u, 0u, 0u};
        }
#pragma unroll
        for (int i = 0; i < BATCH; ++i) {
            const int q = base + i * kIOThreads + t;
            const bool second = q >= per_plane;
            v4u* dst = reinterpret_cast<v4u*>(second ? act_lo : act_hi) + (second ? q - per_plane : q);
            if (q < total) *dst = v[i];
        }
    }
}

// 1/rms of every row from the per-strip sums of squares ss[NSS*4][16]: one wave, NSS loads per
// lane (issued before the copy of the stage input, reduced after it).
template <int NSS>
__device__ __forceinline__ void row_scales_load(const float* ss, int lane, float (&v)[NSS]) {
    const int c = lane & 15, part = lane >> 4;
#pragma unroll
    for (int i = 0; i < NSS; ++i) v[i] = ss[(size_t)(part + 4 * i) * 16 + c];
}
template <int NSS>
__device__ __forceinline__ void row_scales_reduce(const float (&v)[NSS], int K, float eps, int lane, float* rn) {
    float a = 0.f;
#pragma unroll
    for (int i = 0; i < NSS; ++i) a += v[i];
    a = sum_xor16(a);
    a = sum_xor32(a);
    if (lane < 16) rn[lane] = 1.0f / sqrtf(a / (float)K + eps);
}

// Stage the attention output rows for the Wo stage when a head was split into NC chunks:
// merges the chunk partials - softmax statistics (max, sum) and un-normalised outputs.
template <int KREG>
__device__ __forceinline__ void stage_attention(const SP& p, int layer, int io, int lane, uint16_t* act_hi,
                                                uint16_t* act_lo) {
    const float* P = slot(p, layer) + p.o_p;
    const int d = p.d, RS = p.RS, NC = p.NC;
    for (int c = io; c < p.MR; c += kNIO) {
        const int seq = c / RS, r = c - seq * RS;
        float4 o[KREG][kNCMax];
        float2 st[KREG][kNCMax];
#pragma unroll
        for (int i = 0; i < KREG; ++i) {
            const int j = (i * 64 + lane) * 4;
            const int h = j >> 6, dim = j & 63;
#pragma unroll
            for (int cc = 0; cc < kNCMax; ++cc) {
                const bool on = j < d && cc < NC;
                const float* row = P + ((size_t)((seq * p.H + (on ? h : 0)) * NC + (on ? cc : 0)) * RS + r) * kPS;
                o[i][cc] = on ? *reinterpret_cast<const float4*>(row + dim) : make_float4(0.f, 0.f, 0.f, 0.f);
                st[i][cc] = on ? *reinterpret_cast<const float2*>(row + 64) : make_float2(-1e30f, 0.f);
            }
        }
#pragma unroll
        for (int i = 0; i < KREG; ++i) {
            const int j = (i * 64 + lane) * 4;
            if (j < d) {
                float m2 = -1e30f;
#pragma unroll
                for (int cc = 0; cc < kNCMax; ++cc) m2 = fmaxf(m2, st[i][cc].x);
                float dn = 0.f;
                float4 y = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
                for (int cc = 0; cc < kNCMax; ++cc) {
                    const float f = __expf(st[i][cc].x - m2);
                    dn += st[i][cc].y * f;
                    y.x += o[i][cc].x * f; y.y += o[i][cc].y * f; y.z += o[i][cc].z * f; y.w += o[i][cc].w * f;
                }
                const float inv = dn > 0.f ? 1.0f / dn : 0.f;
                y.x *= inv; y.y *= inv; y.z *= inv; y.w *= inv;
                put_split(y, act_hi + (size_t)c * p.Kpd + j, act_lo + (size_t)c * p.Kpd + j);
            }
        }
    }
}

// One wave's MFMAs of a job: strips x its K quarter, activations from LDS.  The B operand of
// a k-tile is shared by every strip of the job, and is fetched two k-tiles ahead.  Columns
// >= MR of the B operand repeat row 0 (their results are never stored); absent strips have
// zero weights.
template <int TPS, int NS>
__device__ __forceinline__ void mfma_job(const v4u (&w)[NS * TPS], int wave, int lane, int MR, const uint16_t* act_hi,
                                         const uint16_t* act_lo, int Kp, f32x4 (&acc)[NS]) {
    const int col = lane & 15, kg = lane >> 4;
    const size_t at = (size_t)(col < MR ? col : 0) * Kp + kg * 8 + (size_t)wave * TPS * 32;
    const uint16_t* bh_base = act_hi + at;
    const uint16_t* bl_base = act_lo + at;
    v4u bh[3], bl[3];
    f32x4 acl[NS];
#pragma unroll
    for (int si = 0; si < NS; ++si) {
        acc[si] = (f32x4){0.f, 0.f, 0.f, 0.f};
        acl[si] = (f32x4){0.f, 0.f, 0.f, 0.f};
    }
#pragma unroll
    for (int j = 0; j < 2 && j < TPS; ++j) {
        bh[j] = *reinterpret_cast<const v4u*>(bh_base + j * 32);
        bl[j] = *reinterpret_cast<const v4u*>(bl_base + j * 32);
    }
#pragma unroll
    for (int j = 0; j < TPS; ++j) {
        if (j + 2 < TPS) {
            bh[(j + 2) % 3] = *reinterpret_cast<const v4u*>(bh_base + (j + 2) * 32);
            bl[(j + 2) % 3] = *reinterpret_cast<const v4u*>(bl_base + (j + 2) * 32);
        }
        const bf16x8 h = __builtin_bit_cast(bf16x8, bh[j % 3]), l = __builtin_bit_cast(bf16x8, bl[j % 3]);
#pragma unroll
        for (int si = 0; si < NS; ++si) {  // hi and lo products accumulate in separate chains
            const bf16x8 a = __builtin_bit_cast(bf16x8, w[si * TPS + j]);
            acc[si] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, h, acc[si], 0, 0, 0);
            acl[si] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, l, acl[si], 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int si = 0; si < NS; ++si) acc[si] += acl[si];
}

// pos: the row's position (rotary angle); slot: its entry in the cache.  Tree rows: node r of the
// candidate tree sits at the root's position plus its depth and in the entry root + r.
struct RowPos { int seq, r, pos, slot; bool valid; };
template <bool TREE = false>
__device__ __forceinline__ RowPos row_pos(const SP& p, int c) {
    RowPos o;
    o.seq = c / p.RS;
    o.r = c - o.seq * p.RS;
    const int b = o.seq % p.B;
    const int ke = p.k_eff[b];
    o.valid = o.r <= ke;
    o.slot = o.valid ? p.C + p.n[b] - 1 + o.r : 0;
    o.pos = o.slot;
    if constexpr (TREE) o.pos = o.valid ? p.C + p.n[b] - 1 + p.tdepth[o.r] : 0;
    return o;
}

// ------------------------------------------------------------------------- GEMV phases

struct Lds {
    uint16_t* act_hi;
    uint16_t* act_lo;
    float* red;      // [kCW][kMaxStrips][64][4]: K-quarter partial strips in accumulator layout
    float* rn;       // [16]: 1/rms of the rows of the stage input
    float* att;      // attention: scaled queries of the job's rows
    unsigned* join;  // arrivals of the IO waves (only ever grows)
};

// Operands of a strip's epilogue that do not depend on this stage, fetched by the strip's IO
// wave before the barrier is crossed.  A lane finishes rows 4*(lane/16)..+3 of column lane%16.
struct EpiPre {
    float2 rot[2];   // stage A: cos, sin of the lane's two rotary pairs
    uint2 gain;      // stages C, E: gain of the following norm for the lane's four rows (bf16 x 4)
};

template <int KIND, bool TREE = false>
__device__ __forceinline__ void epilogue_prefetch(const SP& p, int layer, int strip, int lane, EpiPre& pre) {
    const int c = lane & 15, quad = lane >> 4, d = p.d;
    pre.rot[0] = pre.rot[1] = make_float2(1.f, 0.f);
    pre.gain = make_uint2(0u, 0u);
    if (KIND == K_A) {
        const int o0 = strip * 16, seg = o0 / d, j0 = o0 - seg * d, hd = d / p.H;
        if (c < p.MR && seg < 2) {
            const RowPos rp = row_pos<TREE>(p, c);
            const float2* rt = p.rope + (size_t)rp.pos * (hd / 2) + ((j0 % hd) >> 1) + 2 * quad;
            pre.rot[0] = rt[0];
            pre.rot[1] = rt[1];
        }
    } else if (KIND == K_C || KIND == K_E) {
        const uint16_t* g = KIND == K_C ? p.blob + (p.g2_off + (u64)layer * p.layer_bytes) / 2
                                        : (layer + 1 < p.L ? p.blob + (p.g1_off + (u64)(layer + 1) * p.layer_bytes) / 2
                                                           : p.blob + p.gf_off / 2);
        pre.gain = *reinterpret_cast<const uint2*>(g + strip * 16 + 4 * quad);
    }
}

__device__ __forceinline__ f32x4 times_gain(f32x4 x, uint2 g) {
    return (f32x4){x[0] * bf16_f32(g.x & 0xFFFFu), x[1] * bf16_f32(g.x >> 16), x[2] * bf16_f32(g.y & 0xFFFFu),
                   x[3] * bf16_f32(g.y >> 16)};
}

// Writes a strip of the residual stream for the stage that follows a norm: the values times the
// norm's gain as split planes, and the strip's sum of squares per row.
__device__ __forceinline__ void put_stream(const SP& p, uint16_t* hi, uint16_t* lo, float* ss, int strip, int lane,
                                           f32x4 x, uint2 gain) {
    const int c = lane & 15, quad = lane >> 4;
    const bool live = c < p.MR;
    float s2 = live ? x[0] * x[0] + x[1] * x[1] + x[2] * x[2] + x[3] * x[3] : 0.f;
    s2 = sum_xor16(s2);
    s2 = sum_xor32(s2);
    if (live) {
        const size_t at = (size_t)c * p.Kpd + strip * 16 + 4 * quad;
        st_split4(hi + at, lo + at, times_gain(x, gain));
        if (quad == 0) st_f32(ss + (size_t)strip * 16 + c, s2);
    }
}

// v: the finished strip in accumulator layout (lane: rows 4*(lane/16)..+3 of column lane%16).
template <int KIND, bool TREE = false>
__device__ __forceinline__ void epilogue(const SP& p, const Lds& s, int layer, int strip, f32x4 v, int lane,
                                         const EpiPre& pre, f32x4& resid) {
    const int c = lane & 15, quad = lane >> 4, d = p.d;
    const bool live = c < p.MR;
    if (KIND == K_A) {
        const float r = s.rn[c];
        const int o0 = strip * 16, seg = o0 / d, j0 = o0 - seg * d;
        v *= r;
        const float a0 = v[0] * pre.rot[0].x - v[1] * pre.rot[0].y, b0 = v[0] * pre.rot[0].y + v[1] * pre.rot[0].x;
        const float a1 = v[2] * pre.rot[1].x - v[3] * pre.rot[1].y, b1 = v[2] * pre.rot[1].y + v[3] * pre.rot[1].x;
        if (live) {
            if (seg == 0) {  // queries, already scaled by 1/sqrt(head_dim) = 1/8
                st_f32x4(slot(p, layer) + p.o_q + (size_t)c * d + j0 + 4 * quad,
                         (f32x4){a0 * 0.125f, b0 * 0.125f, a1 * 0.125f, b1 * 0.125f});
            } else {
                const RowPos rp = row_pos<TREE>(p, c);
                if (rp.valid) {
                    // cache layout [layer][sequence][head][position][64]: a strip lies inside one head
                    _Float16* dst = (seg == 1 ? p.Kc : p.Vc) +
                                    ((((size_t)layer * p.Smax + rp.seq) * p.H + j0 / 64) * p.Tmax + rp.slot) * 64 + j0 % 64 + 4 * quad;
                    const _Float16 h0 = (_Float16)a0, h1 = (_Float16)b0, h2 = (_Float16)a1, h3 = (_Float16)b1;
                    st_u64(dst,
                           (unsigned)__builtin_bit_cast(unsigned short, h0) | ((unsigned)__builtin_bit_cast(unsigned short, h1) << 16),
                           (unsigned)__builtin_bit_cast(unsigned short, h2) | ((unsigned)__builtin_bit_cast(unsigned short, h3) << 16));
                }
            }
        }
    } else if (KIND == K_C) {  // x' = x + Wo o
        resid += v;
        put_stream(p, plane(p, layer, p.o_x2h), plane(p, layer, p.o_x2l), slot(p, layer) + p.o_ss2, strip, lane, resid,
                   pre.gain);
    } else if (KIND == K_E) {  // x(next layer) = x' + W2 h
        resid += v;
        put_stream(p, plane(p, layer + 1, p.o_xh), plane(p, layer + 1, p.o_xl), slot(p, layer + 1) + p.o_ssx, strip, lane,
                   resid, pre.gain);
        if (layer == p.L - 1 && live)  // final hidden rows, for the kernels that follow
            *reinterpret_cast<f32x4*>(p.X + (size_t)c * d + strip * 16 + 4 * quad) = resid;
    } else if (KIND == K_D) {  // rows 0..7: W1 rows strip*8+i, rows 8..15: the matching W3 rows
        const float r = s.rn[c];
        v *= r;
        f32x4 u3;
#pragma unroll
        for (int e = 0; e < 4; ++e) u3[e] = lane_xor32(v[e]);
        if (live && quad < 2) {
            f32x4 h;
#pragma unroll
            for (int e = 0; e < 4; ++e) h[e] = v[e] / (1.0f + expf(-v[e])) * u3[e];
            const size_t at = (size_t)c * p.Kpm + strip * 8 + 4 * quad;
            st_split4(plane(p, layer, p.o_hh) + at, plane(p, layer, p.o_hl) + at, h);
        }
    } else if (KIND == K_LM) {
        const float r = s.rn[c];
        if (live) *reinterpret_cast<f32x4*>(p.logit_s + (size_t)c * p.Vs + strip * 16 + 4 * quad) = v * r;
    }
}

// Waits until all IO waves of the workgroup have reached this point (their global stores
// already acknowledged).  LDS only; bounded like the grid barrier.
__device__ __forceinline__ void io_join(const Lds& s, Barrier& bar, int lane) {
    const unsigned want = ++bar.joins * kNIO;
    if (lane == 0) atomicAdd(s.join, 1u);
    for (unsigned spins = 0; spins < kSpinLimit; ++spins) {
        if ((int)(__hip_atomic_load(s.join, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) - want) >= 0) break;
        __builtin_amdgcn_s_sleep(1);
    }
    compiler_fence();
}

// The IO waves' end of a stage: stores acknowledged, all IO waves joined, one arrival posted.
__device__ __forceinline__ void io_finish(const SP& p, const Lds& s, Barrier& bar, unsigned ph, int wave, int lane) {
    __builtin_amdgcn_s_waitcnt(0);
    io_join(s, bar, lane);
    stamp(p, ph, 5);
    stamp_all(p, ph, 0);
    const bool poster = wave == kCW && lane == 0;
    unsigned prev = 0u;
    if (poster) prev = bar.arrive_issue();
    __builtin_amdgcn_s_barrier();  // pairs with compute_finish: the next stage's loads queue behind the arrival
    if (poster) bar.arrive_finish(prev); else ++bar.id;
    stamp(p, ph, 6);
}

// The compute waves' end of a stage: they go on to request the next stage's weights only once
// this stage's results are acknowledged and its arrival has been sent, so that neither waits in
// the compute unit's memory pipeline behind a hundred KB of prefetch.
__device__ __forceinline__ void compute_finish(Barrier& bar) {
    __builtin_amdgcn_s_barrier();
    ++bar.id;
}

// First stage of a launch: the owners of the residual strips pick their slice of the embedded
// rows up and publish it in the form stage A of layer 0 expects.
__device__ __forceinline__ void prologue_phase(const SP& p, const Lds& s, Barrier& bar, f32x4& resid) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const Job job = load_job(p, K_C, 0, 0);
    const unsigned ph = bar.id - bar.first;
    if (wave >= kCW) {
        stamp(p, ph, 0);
        if (wave == kCW && job.nstrips) {
            const int c = lane & 15, quad = lane >> 4, strip = job.strip[0];
            const uint2 gain = *reinterpret_cast<const uint2*>(p.blob + p.g1_off / 2 + strip * 16 + 4 * quad);
            resid = c < p.MR ? *reinterpret_cast<const f32x4*>(p.X + (size_t)c * p.d + strip * 16 + 4 * quad)
                             : (f32x4){0.f, 0.f, 0.f, 0.f};
            put_stream(p, plane(p, 0, p.o_xh), plane(p, 0, p.o_xl), slot(p, 0) + p.o_ssx, strip, lane, resid, gain);
        }
        io_finish(p, s, bar, ph, wave, lane);
    } else {
        compute_finish(bar);
    }
}

// ---- draft head (Method, spatial draft head: g_i = W_d [g_{i-1} | E[left] | E[up]], then the
// target's final norm and output projection).  W_d is streamed as three [d, d] column blocks.

// Stage the input of column block `blk` for every sequence: the previous hidden state (fp32,
// split here), or the embedding row of the left / upper neighbour (bf16: its own hi part).
template <int KREG>
__device__ __forceinline__ void stage_draft_input(const SP& p, int blk, int io, int lane, uint16_t* act_hi, uint16_t* act_lo) {
    const int d = p.d, i = p.step_i;
    const uint16_t* E = p.blob + p.E_off / 2;
    for (int c = io; c < p.MR; c += kNIO) {
        const int b = c % p.B;
        const bool valid = i <= p.k_eff[b];
        const int n = p.n[b], t = n - 1 + i;
        int tok = -1;
        if (valid && blk == 1) tok = (i == 1) ? p.grid[(size_t)b * p.N + n - 1] : p.draft[b * p.kstride + i - 2];
        if (valid && blk == 2 && t >= p.IW) tok = p.grid[(size_t)b * p.N + t - p.IW];
#pragma unroll
        for (int q = 0; q < KREG; ++q) {
            const int j = (q * 64 + lane) * 4;
            if (j < d) {
                uint16_t* hi = act_hi + (size_t)c * p.Kpd + j;
                uint16_t* lo = act_lo + (size_t)c * p.Kpd + j;
                if (blk == 0) {
                    const float4 v = valid ? *reinterpret_cast<const float4*>(p.prev + (size_t)c * d + j)
                                           : make_float4(0.f, 0.f, 0.f, 0.f);
                    put_split(v, hi, lo);
                } else {
                    *reinterpret_cast<uint2*>(hi) = tok >= 0 ? *reinterpret_cast<const uint2*>(E + (size_t)tok * d + j)
                                                            : make_uint2(0u, 0u);
                    *reinterpret_cast<uint2*>(lo) = make_uint2(0u, 0u);
                }
            }
        }
    }
}

// Stage the head's output for the output projection: g = sum of the three block partials,
// times the final norm's gain, split; 1/rms per row; workgroup 0 also keeps g itself.
template <int KREG>
__device__ __forceinline__ void stage_head_output(const SP& p, int io, int lane, const Lds& s) {
    const int d = p.d;
    const uint16_t* gain = p.blob + p.gf_off / 2;
    for (int c = io; c < p.MR; c += kNIO) {
        float4 g[KREG];
        float ss = 0.f;
#pragma unroll
        for (int q = 0; q < KREG; ++q) {
            const int j = (q * 64 + lane) * 4;
            g[q] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (j < d) {
                const float4 a = *reinterpret_cast<const float4*>(p.dpart + ((size_t)(0 * 16 + c)) * d + j);
                const float4 b = *reinterpret_cast<const float4*>(p.dpart + ((size_t)(1 * 16 + c)) * d + j);
                const float4 e = *reinterpret_cast<const float4*>(p.dpart + ((size_t)(2 * 16 + c)) * d + j);
                g[q] = make_float4(a.x + b.x + e.x, a.y + b.y + e.y, a.z + b.z + e.z, a.w + b.w + e.w);
                ss += g[q].x * g[q].x + g[q].y * g[q].y + g[q].z * g[q].z + g[q].w * g[q].w;
            }
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o, 64);
        if (lane == 0) s.rn[c] = 1.0f / sqrtf(ss / (float)d + p.eps);
#pragma unroll
        for (int q = 0; q < KREG; ++q) {
            const int j = (q * 64 + lane) * 4;
            if (j < d) {
                const uint2 gn = *reinterpret_cast<const uint2*>(gain + j);
                const float4 y = make_float4(g[q].x * bf16_f32(gn.x & 0xFFFFu), g[q].y * bf16_f32(gn.x >> 16),
                                             g[q].z * bf16_f32(gn.y & 0xFFFFu), g[q].w * bf16_f32(gn.y >> 16));
                put_split(y, s.act_hi + (size_t)c * p.Kpd + j, s.act_lo + (size_t)c * p.Kpd + j);
                if (blockIdx.x == 0) *reinterpret_cast<float4*>(p.gout + (size_t)c * d + j) = g[q];
            }
        }
    }
}

// KIND: which matrix; TPS: k-tiles per compute wave and strip; NSS: per-strip sums of squares
// per lane of the row-scale reduction (0: the stage input is not normalised); BATCH: chunks in
// flight per IO thread while copying the stage input.
template <int KIND, int TPS, int NSS, int BATCH, int KREG, int STAGE = 0, bool TREE = false>
__device__ __forceinline__ void gemv_phase(const SP& p, const Lds& s, Barrier& bar, int layer, int round,
                                           const uint16_t* src_hi, const uint16_t* src_lo, const float* ss, int K, int Kp,
                                           f32x4& resid) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const bool is_io = wave >= kCW;
    const Job job = load_job(p, KIND, round, layer);
    const unsigned ph = bar.id - bar.first + (KIND == K_LM ? round : 0);
    // The rounds of the output projection share one input: only the first waits and stages it.
    const bool fresh = !(KIND == K_LM && round > 0);
    // Nothing in this block depends on the previous stage, so it is requested before the barrier
    // is crossed: the weights (compute waves), rotary factors and gains (IO waves).
    constexpr int NS = kTMax / TPS < kMaxStrips ? kTMax / TPS : kMaxStrips;  // strips a job of this kind can have
    v4u w[NS * TPS];
    EpiPre pre;
    if (!is_io) {
        stamp_c(p, ph, 0);
        issue_tiles<TPS, NS>(p, job, wave, lane, w);
        stamp_c(p, ph, 1);
    } else {
        stamp(p, ph, 0);
        if (wave - kCW < job.nstrips) epilogue_prefetch<KIND, TREE>(p, layer, job.strip[wave - kCW], lane, pre);
        if (fresh) {
            bar.wait();
            stamp(p, ph, 1);
            stamp_all(p, ph, 1);
            float ssv[NSS > 0 ? NSS : 1];
            if constexpr (NSS > 0) {
                if (wave == kCW + kNIO - 1) row_scales_load<NSS>(ss, lane, ssv);
            }
            if constexpr (STAGE == 1) {
                stage_head_output<KREG>(p, wave - kCW, lane, s);
            } else if (KIND == K_C && p.NC > 1) {
                if (job.nstrips) stage_attention<KREG>(p, layer, wave - kCW, lane, s.act_hi, s.act_lo);
            } else if (job.nstrips || KIND == K_LM) {
                stage_copy<BATCH>(src_hi, src_lo, p.MR, Kp, s.act_hi, s.act_lo, threadIdx.x - kCW * 64);
            }
            if constexpr (NSS > 0) {
                if (wave == kCW + kNIO - 1) row_scales_reduce<NSS>(ssv, K, p.eps, lane, s.rn);
            }
        }
        stamp(p, ph, 2);
    }
    __syncthreads();
    stamp(p, ph, 3);
    if (!is_io && job.nstrips) {
        stamp_c(p, ph, 2);
        if (p.dbg) { __builtin_amdgcn_s_waitcnt(0); stamp_c(p, ph, 3); }
        f32x4 acc[NS];
        mfma_job<TPS, NS>(w, wave, lane, p.MR, s.act_hi, s.act_lo, Kp, acc);
        stamp_c(p, ph, 4);
#pragma unroll
        for (int i = 0; i < NS; ++i)
            *reinterpret_cast<f32x4*>(s.red + (((size_t)wave * kMaxStrips + i) * 64 + lane) * 4) = acc[i];
        stamp_c(p, ph, 5);
    }
    __syncthreads();
    stamp(p, ph, 4);
    if (is_io) {
        const int i = wave - kCW;  // IO wave i finishes strip i of the job
        if (i < job.nstrips) {
            f32x4 v = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int cw = 0; cw < kCW; ++cw)
                v += *reinterpret_cast<const f32x4*>(s.red + (((size_t)cw * kMaxStrips + i) * 64 + lane) * 4);
            epilogue<KIND, TREE>(p, s, layer, job.strip[i], v, lane, pre, resid);
        }
    }
    if (is_io) {
        if (KIND != K_LM) io_finish(p, s, bar, ph, wave, lane);  // nothing follows the output projection
    } else if (KIND != K_LM) {
        compute_finish(bar);
    }
}

// Stage E (W2): `esplit` workgroups share a strip, each with its own K range.  Part 0 owns the
// strip's residual; the others hand it their partial sums through words that read 0xFFFFFFFF
// until written (a NaN pattern no sum can produce; the owner restores it after reading), so the
// hand-over costs one store -> poll trip instead of a grid barrier.
template <int TPS, int BATCH>
__device__ __forceinline__ void w2_phase(const SP& p, const Lds& s, Barrier& bar, int layer, f32x4& resid) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const bool is_io = wave >= kCW;
    const Job job = load_job(p, K_E, 0, layer);
    const int strip = job.strip[0], part = job.strip[1];
    const unsigned ph = bar.id - bar.first;
    constexpr int KPART = TPS * kCW * 32;        // K range of one part
    constexpr int CPR = KPART / 8;               // 16-byte chunks per row of it
    v4u w[TPS];
    EpiPre pre;
    if (!is_io) {
        issue_tiles<TPS, 1>(p, job, wave, lane, w);
    } else {
        stamp(p, ph, 0);
        if (wave == kCW && job.nstrips && part == 0) epilogue_prefetch<K_E>(p, layer, strip, lane, pre);
        bar.wait();
        stamp(p, ph, 1);
        stamp_all(p, ph, 1);
        if (job.nstrips) {  // copy the part's columns of the split planes: chunk q = (plane, row, column chunk)
            const int t = threadIdx.x - kCW * 64, total = 2 * p.MR * CPR;
            const uint16_t* hi = plane(p, layer, p.o_hh) + (size_t)part * KPART;
            const uint16_t* lo = plane(p, layer, p.o_hl) + (size_t)part * KPART;
            for (int base = 0; base < total; base += BATCH * kIOThreads) {
                v4u v[BATCH];
#pragma unroll
                for (int i = 0; i < BATCH; ++i) {
                    const int q = base + i * kIOThreads + t, pr = q / CPR, j8 = q - pr * CPR;
                    const int c = pr >= p.MR ? pr - p.MR : pr;
                    const uint16_t* src = (pr >= p.MR ? lo : hi) + (size_t)c * p.Kpm + j8 * 8;
                    v[i] = q < total ? *reinterpret_cast<const v4u*>(src) : (v4u){0u, 0u, 0u, 0u};
                }
#pragma unroll
                for (int i = 0; i < BATCH; ++i) {
                    const int q = base + i * kIOThreads + t, pr = q / CPR, j8 = q - pr * CPR;
                    const int c = pr >= p.MR ? pr - p.MR : pr;
                    uint16_t* dst = (pr >= p.MR ? s.act_lo : s.act_hi) + (size_t)c * p.KpE + j8 * 8;
                    if (q < total) *reinterpret_cast<v4u*>(dst) = v[i];
                }
            }
        }
        stamp(p, ph, 2);
    }
    __syncthreads();
    stamp(p, ph, 3);
    if (!is_io && job.nstrips) {
        f32x4 acc[1];
        mfma_job<TPS, 1>(w, wave, lane, p.MR, s.act_hi, s.act_lo, p.KpE, acc);
        *reinterpret_cast<f32x4*>(s.red + (((size_t)wave * kMaxStrips) * 64 + lane) * 4) = acc[0];
    }
    __syncthreads();
    stamp(p, ph, 4);
    if (wave == kCW && job.nstrips) {
        f32x4 v = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int cw = 0; cw < kCW; ++cw)
            v += *reinterpret_cast<const f32x4*>(s.red + (((size_t)cw * kMaxStrips) * 64 + lane) * 4);
        float* mail = slot(p, layer) + p.o_ep + ((size_t)strip * (p.esplit - 1)) * 256 + lane * 4;
        if (part > 0) {
            st_f32x4(mail + (size_t)(part - 1) * 256, v);
        } else {
            for (int j = 0; j + 1 < p.esplit; ++j) {
                u64* src = reinterpret_cast<u64*>(mail + (size_t)j * 256);
                u64 a = ~0ull, b = ~0ull;
                bool ok = false;
                for (unsigned spins = 0; spins < kSpinLimit && !ok; ++spins) {
                    a = __hip_atomic_load(src, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    b = __hip_atomic_load(src + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    ok = (unsigned)a != ~0u && (unsigned)(a >> 32) != ~0u && (unsigned)b != ~0u && (unsigned)(b >> 32) != ~0u;
                    ok = __all(ok);  // the wave leaves the loop together
                    if (!ok && (spins & 255u) == 255u &&
                        __hip_atomic_load(p.err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u) break;
                }
                if (!ok) __hip_atomic_store(p.err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                v += (f32x4){__uint_as_float((unsigned)a), __uint_as_float((unsigned)(a >> 32)),
                             __uint_as_float((unsigned)b), __uint_as_float((unsigned)(b >> 32))};
                __hip_atomic_store(src, ~0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);      // "not written yet" again
                __hip_atomic_store(src + 1, ~0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            epilogue<K_E>(p, s, layer, strip, v, lane, pre, resid);
        }
    }
    if (is_io) io_finish(p, s, bar, ph, wave, lane);
    else compute_finish(bar);
}

// ------------------------------------------------------------------------- attention

// A job = (sequence, head, row group, chunk): it reduces its slice of the cached positions -
// requested before the barrier is crossed, they were written by earlier launches - and, for the
// last chunk, the rows appended by this launch, for the query rows of its group.
// Lane layout: 8 positions per wave load, 8 lanes x 8 dims per position.
struct AttnAcc {
    float acc[8], mx, den;
};

// Sum over the 8 lanes that share a cache position (cross-lane moves in the VALU, no LDS).
__device__ __forceinline__ float sum8(float v) {
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xB1, 0xF, 0xF, true));   // quad_perm [1,0,3,2]
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x4E, 0xF, 0xF, true));   // quad_perm [2,3,0,1]
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x141, 0xF, 0xF, true));  // row_half_mirror
    return v;
}

__device__ __forceinline__ void halves8(v4u raw, float (&f)[8]) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        f[2 * e] = (float)__builtin_bit_cast(_Float16, (unsigned short)(raw[e] & 0xFFFFu));
        f[2 * e + 1] = (float)__builtin_bit_cast(_Float16, (unsigned short)(raw[e] >> 16));
    }
}

// One cache position per lane group.  q: the lane's 8 dims of the job's scaled query rows; r0:
// absolute index of the first row; row_lo: first absolute row that may see the position; ke:
// last valid row.
template <int RPJ>
__device__ __forceinline__ void attend(const float (&q)[RPJ][8], int r0, v4u kraw, v4u vraw, int row_lo, int ke,
                                       AttnAcc (&A)[RPJ]) {
    float kf[8], vf[8];
    halves8(kraw, kf);
    halves8(vraw, vf);
#pragma unroll
    for (int r = 0; r < RPJ; ++r) {
        float sc = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) sc += q[r][e] * kf[e];
        sc = sum8(sc);
        if (r0 + r >= row_lo && r0 + r <= ke) {
            const float mn = fmaxf(A[r].mx, sc);
            const float corr = __expf(A[r].mx - mn), pw = __expf(sc - mn);
            A[r].den = A[r].den * corr + pw;
#pragma unroll
            for (int e = 0; e < 8; ++e) A[r].acc[e] = A[r].acc[e] * corr + pw * vf[e];
            A[r].mx = mn;
        }
    }
}

// The same for tree rows: bit r of vis says whether absolute row r sees the position.
template <int RPJ>
__device__ __forceinline__ void attend_vis(const float (&q)[RPJ][8], int r0, v4u kraw, v4u vraw, unsigned vis, int ke,
                                           AttnAcc (&A)[RPJ]) {
    float kf[8], vf[8];
    halves8(kraw, kf);
    halves8(vraw, vf);
#pragma unroll
    for (int r = 0; r < RPJ; ++r) {
        float sc = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) sc += q[r][e] * kf[e];
        sc = sum8(sc);
        if (((vis >> (r0 + r)) & 1u) && r0 + r <= ke) {
            const float mn = fmaxf(A[r].mx, sc);
            const float corr = __expf(A[r].mx - mn), pw = __expf(sc - mn);
            A[r].den = A[r].den * corr + pw;
#pragma unroll
            for (int e = 0; e < 8; ++e) A[r].acc[e] = A[r].acc[e] * corr + pw * vf[e];
            A[r].mx = mn;
        }
    }
}

// kNIT cache positions per lane group at once (positions pos0 + it * stride, those < o1 count):
// all scores first, one running-maximum update per row, then the weighted values - independent
// work for the VALU instead of one dependent chain per position.
template <int RPJ>
__device__ __forceinline__ void attend_round(const float (&q)[RPJ][8], int r0, const v4u (&kk)[kNIT], const v4u (&vv)[kNIT],
                                             int pos0, int stride, int o1, int ke, AttnAcc (&A)[RPJ]) {
    float sc[RPJ][kNIT];
#pragma unroll
    for (int it = 0; it < kNIT; ++it) {
        float kf[8];
        halves8(kk[it], kf);
        const bool on = pos0 + it * stride < o1;
#pragma unroll
        for (int r = 0; r < RPJ; ++r) {
            float d = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) d += q[r][e] * kf[e];
            d = sum8(d);
            sc[r][it] = (on && r0 + r <= ke) ? d : -1e30f;
        }
    }
#pragma unroll
    for (int r = 0; r < RPJ; ++r) {
        float mn = A[r].mx;
#pragma unroll
        for (int it = 0; it < kNIT; ++it) mn = fmaxf(mn, sc[r][it]);
        const float corr = __expf(A[r].mx - mn);
        float sum = 0.f;
#pragma unroll
        for (int it = 0; it < kNIT; ++it) {
            sc[r][it] = sc[r][it] > -1e29f ? __expf(sc[r][it] - mn) : 0.f;
            sum += sc[r][it];
        }
        A[r].den = A[r].den * corr + sum;
        A[r].mx = mn;
#pragma unroll
        for (int e = 0; e < 8; ++e) A[r].acc[e] *= corr;
    }
#pragma unroll
    for (int it = 0; it < kNIT; ++it) {
        float vf[8];
        halves8(vv[it], vf);
#pragma unroll
        for (int r = 0; r < RPJ; ++r)
#pragma unroll
            for (int e = 0; e < 8; ++e) A[r].acc[e] += sc[r][it] * vf[e];
    }
}

template <int RPJ, bool TREE = false>
__device__ __forceinline__ void attn_phase(const SP& p, const Lds& s, Barrier& bar, int layer) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const bool is_io = wave >= kCW;
    // Jobs of one (sequence, head) sit on one XCD, so that its L2 serves their common K/V rows.
    const int xcd = blockIdx.x % kXcd, li = blockIdx.x / kXcd, per = p.NRG * p.NC;
    const int sh = xcd + kXcd * (li / per), sub = li % per;
    const bool have = sh < p.S * p.H;
    const int seq = have ? sh / p.H : 0, h = have ? sh % p.H : 0, rg = sub / p.NC, ch = sub % p.NC;
    const int d = p.d, RS = p.RS, r0 = rg * RPJ;
    float* qs = s.att;                                   // [RPJ][64] scaled queries
    float* part = reinterpret_cast<float*>(s.act_hi);    // [kCW][RPJ][kPS], over the idle activation buffers
    const unsigned ph = bar.id - bar.first;
    const int pg = lane >> 3, dg = lane & 7;
    const int b = seq % p.B;
    const int ke = have ? p.k_eff[b] : -1;
    const int kv0 = ke >= 0 ? p.C + p.n[b] - 1 : 0;  // positions cached before this launch
    const int o0 = (int)((long long)kv0 * ch / p.NC), o1 = (int)((long long)kv0 * (ch + 1) / p.NC);
    const int nrounds = (o1 - o0 + kNIT * kCW * 8 - 1) / (kNIT * kCW * 8);
    const size_t base = ((((size_t)layer * p.Smax + seq) * p.H + h) * p.Tmax) * 64 + dg * 8;   // this head's entries, contiguous
    v4u ka[kNIT], va[kNIT], kb[kNIT], vb[kNIT];
    auto fetch = [&](v4u (&kk)[kNIT], v4u (&vv)[kNIT], int rnd) {
#pragma unroll
        for (int it = 0; it < kNIT; ++it) {
            const int pos = o0 + (rnd * kNIT + it) * (kCW * 8) + wave * 8 + pg;
            if (pos < o1) {
                kk[it] = *reinterpret_cast<const v4u*>(p.Kc + base + (size_t)pos * 64);
                vv[it] = *reinterpret_cast<const v4u*>(p.Vc + base + (size_t)pos * 64);
            } else {
                kk[it] = (v4u){0u, 0u, 0u, 0u};
                vv[it] = (v4u){0u, 0u, 0u, 0u};
            }
        }
    };
    if (!is_io && have) {
        stamp_c(p, ph, 0);
        fetch(ka, va, 0);
        fetch(kb, vb, 1);
        stamp_c(p, ph, 1);
    }
    if (is_io) {
        stamp(p, ph, 0);
        bar.wait();
        stamp(p, ph, 1);
        stamp_all(p, ph, 1);
        if (have && wave == kCW)
            for (int r = 0; r < RPJ; ++r)
                qs[r * 64 + lane] = r0 + r < RS ? (slot(p, layer) + p.o_q)[(size_t)(seq * RS + r0 + r) * d + h * 64 + lane] : 0.f;
        stamp(p, ph, 2);
    }
    __syncthreads();
    stamp(p, ph, 3);
    if (!is_io && have) {
        stamp_c(p, ph, 2);
        AttnAcc A[RPJ];
#pragma unroll
        for (int r = 0; r < RPJ; ++r) {
            A[r].mx = -1e30f; A[r].den = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) A[r].acc[e] = 0.f;
        }
        float q[RPJ][8];  // the lane's dims of the job's query rows
#pragma unroll
        for (int r = 0; r < RPJ; ++r) {
            const float4 qa = *reinterpret_cast<const float4*>(qs + r * 64 + dg * 8);
            const float4 qb = *reinterpret_cast<const float4*>(qs + r * 64 + dg * 8 + 4);
            q[r][0] = qa.x; q[r][1] = qa.y; q[r][2] = qa.z; q[r][3] = qa.w;
            q[r][4] = qb.x; q[r][5] = qb.y; q[r][6] = qb.z; q[r][7] = qb.w;
        }
        auto run = [&](const v4u (&kk)[kNIT], const v4u (&vv)[kNIT], int rnd) {
            const int pos0 = o0 + rnd * kNIT * (kCW * 8) + wave * 8 + pg;
            attend_round<RPJ>(q, r0, kk, vv, pos0, kCW * 8, o1, ke, A);
        };
        for (int rnd = 0; rnd < nrounds; rnd += 2) {
            run(ka, va, rnd);
            fetch(ka, va, rnd + 2);
            run(kb, vb, rnd + 1);
            fetch(kb, vb, rnd + 3);
        }
        stamp_c(p, ph, 3);
        if constexpr (TREE) {
            // entries appended by this launch (node a in entry kv0 + a, up to 16 of them): a row
            // sees its ancestors' and its own
            if (ch == p.NC - 1 && wave == 0) {
                for (int a = pg; a <= ke; a += 8) {
                    const _Float16* kp = p.Kc + base + (size_t)(kv0 + a) * 64;
                    const _Float16* vp = p.Vc + base + (size_t)(kv0 + a) * 64;
                    const u64 a0 = __hip_atomic_load(reinterpret_cast<const u64*>(kp), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    const u64 a1 = __hip_atomic_load(reinterpret_cast<const u64*>(kp) + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    const u64 b0 = __hip_atomic_load(reinterpret_cast<const u64*>(vp), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    const u64 b1 = __hip_atomic_load(reinterpret_cast<const u64*>(vp) + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    const v4u kraw = (v4u){(unsigned)a0, (unsigned)(a0 >> 32), (unsigned)a1, (unsigned)(a1 >> 32)};
                    const v4u vraw = (v4u){(unsigned)b0, (unsigned)(b0 >> 32), (unsigned)b1, (unsigned)(b1 >> 32)};
                    unsigned vis = 0u;
#pragma unroll
                    for (int r = 0; r < RPJ; ++r) {
                        const int row = r0 + r;
                        if (row < RS && (row == a || ((p.tanc[row] >> a) & 1ull))) vis |= 1u << row;
                    }
                    attend_vis<RPJ>(q, r0, kraw, vraw, vis, ke, A);
                }
            }
        } else
        if (ch == p.NC - 1 && wave == 0 && pg <= ke) {  // rows appended by this launch: coherent loads
            const _Float16* kp = p.Kc + base + (size_t)(kv0 + pg) * 64;
            const _Float16* vp = p.Vc + base + (size_t)(kv0 + pg) * 64;
            const u64 a0 = __hip_atomic_load(reinterpret_cast<const u64*>(kp), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const u64 a1 = __hip_atomic_load(reinterpret_cast<const u64*>(kp) + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const u64 b0 = __hip_atomic_load(reinterpret_cast<const u64*>(vp), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const u64 b1 = __hip_atomic_load(reinterpret_cast<const u64*>(vp) + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const v4u kraw = (v4u){(unsigned)a0, (unsigned)(a0 >> 32), (unsigned)a1, (unsigned)(a1 >> 32)};
            const v4u vraw = (v4u){(unsigned)b0, (unsigned)(b0 >> 32), (unsigned)b1, (unsigned)(b1 >> 32)};
            attend<RPJ>(q, r0, kraw, vraw, pg, ke, A);  // row r sees appended row pg iff pg <= r
        }
        stamp_c(p, ph, 4);
        // merge the eight position groups of the wave (lanes that share dg), then hand the wave's
        // partial to the IO waves through LDS: part[wave][row][kPS]
#pragma unroll
        for (int r = 0; r < RPJ; ++r) {
#pragma unroll
            for (int o = 8; o < 64; o <<= 1) {
                auto other = [&](float x) { return o == 8 ? lane_xor8(x) : (o == 16 ? lane_xor16(x) : lane_xor32(x)); };
                const float omx = other(A[r].mx), oden = other(A[r].den);
                const float mn = fmaxf(A[r].mx, omx);
                const float f0 = __expf(A[r].mx - mn), f1 = __expf(omx - mn);
                A[r].den = A[r].den * f0 + oden * f1;
#pragma unroll
                for (int e = 0; e < 8; ++e) A[r].acc[e] = A[r].acc[e] * f0 + other(A[r].acc[e]) * f1;
                A[r].mx = mn;
            }
            if (pg == 0) {
                float* mine = part + ((size_t)wave * RPJ + r) * kPS;
                *reinterpret_cast<float4*>(mine + dg * 8) = make_float4(A[r].acc[0], A[r].acc[1], A[r].acc[2], A[r].acc[3]);
                *reinterpret_cast<float4*>(mine + dg * 8 + 4) = make_float4(A[r].acc[4], A[r].acc[5], A[r].acc[6], A[r].acc[7]);
                if (dg == 0) *reinterpret_cast<float2*>(mine + 64) = make_float2(A[r].mx, A[r].den);
            }
        }
    }
    if (!is_io && have) stamp_c(p, ph, 5);
    __syncthreads();
    stamp(p, ph, 4);
    if (is_io) {
        const int t = threadIdx.x - kCW * 64;  // thread t: row t / 16 of the job, output dims 4 * (t % 16)..+3
        const int r = t >> 4, q4 = t & 15;
        if (have && r < RPJ && r0 + r < RS) {
            float m2 = -1e30f;
#pragma unroll
            for (int w = 0; w < kCW; ++w) m2 = fmaxf(m2, part[((size_t)w * RPJ + r) * kPS + 64]);
            float dn = 0.f;
            f32x4 o = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int w = 0; w < kCW; ++w) {
                const float* src = part + ((size_t)w * RPJ + r) * kPS;
                const float f = __expf(src[64] - m2);
                dn += src[65] * f;
                o += *reinterpret_cast<const f32x4*>(src + 4 * q4) * f;
            }
            if (p.NC == 1) {  // finished rows of the head: normalise and publish split
                const float inv = dn > 0.f ? 1.0f / dn : 0.f;
                const size_t at = (size_t)(seq * RS + r0 + r) * p.Kpd + h * 64 + 4 * q4;
                st_split4(plane(p, layer, p.o_oh) + at, plane(p, layer, p.o_ol) + at, o * inv);
            } else {
                float* out = slot(p, layer) + p.o_p + ((size_t)(sh * p.NC + ch) * RS + r0 + r) * kPS;
                st_f32x4(out + 4 * q4, o);
                if (q4 == 0) st_f32x2(out + 64, m2, dn);
            }
        }
    }
    if (is_io) {
        io_finish(p, s, bar, ph, wave, lane);
    } else {
        compute_finish(bar);
    }
}

// ------------------------------------------------------------------------- the kernel

// TREE: the rows are the nodes of a candidate tree, TRPJ of them per attention job.
template <int TPS_D, int TPS_M, int KREG_D, int RSMAX, bool TREE = false, int TRPJ = 2>
__global__ __launch_bounds__(kThreads, 1) void verify_stream_kernel(SP p) {
    extern __shared__ uint4 smem_raw[];
    Lds s;
    s.act_hi = reinterpret_cast<uint16_t*>(smem_raw);
    s.act_lo = s.act_hi + (size_t)(p.act_bytes / 4);
    s.red = reinterpret_cast<float*>(reinterpret_cast<char*>(smem_raw) + p.act_bytes);
    s.rn = s.red + kCW * kMaxStrips * 64 * 4;
    s.att = s.rn + 16;
    s.join = reinterpret_cast<unsigned*>(s.att + RSMAX * 64);
    if (threadIdx.x == 0) *s.join = 0u;
    __syncthreads();
    Barrier bar;
    bar.mem = p.bar; bar.err = p.err; bar.id = p.epoch0; bar.first = p.epoch0; bar.joins = 0; bar.dead = false;
    f32x4 resid = (f32x4){0.f, 0.f, 0.f, 0.f};  // the workgroup's strip of the residual stream (first IO wave)
    constexpr int NSS = 2 * TPS_D;             // (d / 16 strips) / 4 lane groups
    prologue_phase(p, s, bar, resid);
    for (int l = 0; l < p.L; ++l) {
        gemv_phase<K_A, TPS_D, NSS, 8, KREG_D, 0, TREE>(p, s, bar, l, 0, plane(p, l, p.o_xh), plane(p, l, p.o_xl),
                                                        slot(p, l) + p.o_ssx, p.d, p.Kpd, resid);
        attn_phase<TREE ? TRPJ : 1, TREE>(p, s, bar, l);
        gemv_phase<K_C, TPS_D, 0, 8, KREG_D>(p, s, bar, l, 0, plane(p, l, p.o_oh), plane(p, l, p.o_ol), nullptr, p.d,
                                             p.Kpd, resid);
        gemv_phase<K_D, TPS_D, NSS, 8, KREG_D>(p, s, bar, l, 0, plane(p, l, p.o_x2h), plane(p, l, p.o_x2l),
                                               slot(p, l) + p.o_ss2, p.d, p.Kpd, resid);
        w2_phase<TPS_M, (2 * 6 * TPS_M * kCW * 4 + kIOThreads - 1) / kIOThreads>(p, s, bar, l, resid);
    }
    for (int r = 0; r < p.rounds[K_LM]; ++r)
        gemv_phase<K_LM, TPS_D, NSS, 8, KREG_D>(p, s, bar, p.L - 1, r, plane(p, p.L, p.o_xh), plane(p, p.L, p.o_xl),
                                                slot(p, p.L) + p.o_ssx, p.d, p.Kpd, resid);
}

// One draft micro-step up to the logits (the sampling kernel follows): stage W (three column
// blocks of W_d over 3 d/16 strips), one grid barrier, then the output projection.
template <int TPS_D, int KREG_D, int RSMAX>
__global__ __launch_bounds__(kThreads, 1) void draft_stream_kernel(SP p) {
    extern __shared__ uint4 smem_raw[];
    Lds s;
    s.act_hi = reinterpret_cast<uint16_t*>(smem_raw);
    s.act_lo = s.act_hi + (size_t)(p.act_bytes / 4);
    s.red = reinterpret_cast<float*>(reinterpret_cast<char*>(smem_raw) + p.act_bytes);
    s.rn = s.red + kCW * kMaxStrips * 64 * 4;
    s.att = s.rn + 16;
    s.join = reinterpret_cast<unsigned*>(s.att + RSMAX * 64);
    if (threadIdx.x == 0) *s.join = 0u;
    __syncthreads();
    Barrier bar;
    bar.mem = p.bar; bar.err = p.err; bar.id = p.epoch0; bar.first = p.epoch0; bar.joins = 0; bar.dead = false;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const bool is_io = wave >= kCW;
    {
        constexpr int NS = kTMax / TPS_D < kMaxStrips ? kTMax / TPS_D : kMaxStrips;
        const Job job = load_job(p, K_WD, 0, 0);
        const unsigned ph = 0;
        const int per = p.d / 16, blk = job.nstrips ? job.strip[0] / per : 0, sl = job.nstrips ? job.strip[0] - blk * per : 0;
        v4u w[NS * TPS_D];
        if (!is_io) {
            issue_tiles<TPS_D, NS>(p, job, wave, lane, w);
        } else {
            stamp(p, ph, 0);
            if (job.nstrips) stage_draft_input<KREG_D>(p, blk, wave - kCW, lane, s.act_hi, s.act_lo);
            stamp(p, ph, 2);
        }
        __syncthreads();
        if (!is_io && job.nstrips) {
            f32x4 acc[NS];
            mfma_job<TPS_D, NS>(w, wave, lane, p.MR, s.act_hi, s.act_lo, p.Kpd, acc);
            *reinterpret_cast<f32x4*>(s.red + (((size_t)wave * kMaxStrips) * 64 + lane) * 4) = acc[0];
        }
        __syncthreads();
        stamp(p, ph, 4);
        if (wave == kCW && job.nstrips) {
            f32x4 v = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int cw = 0; cw < kCW; ++cw)
                v += *reinterpret_cast<const f32x4*>(s.red + (((size_t)cw * kMaxStrips) * 64 + lane) * 4);
            const int c = lane & 15, quad = lane >> 4;
            if (c < p.MR) st_f32x4(p.dpart + ((size_t)(blk * 16 + c)) * p.d + sl * 16 + 4 * quad, v);
        }
        if (is_io) io_finish(p, s, bar, ph, wave, lane);
        else compute_finish(bar);
    }
    f32x4 resid = (f32x4){0.f, 0.f, 0.f, 0.f};
    for (int r = 0; r < p.rounds[K_LM]; ++r)
        gemv_phase<K_LM, TPS_D, 0, 8, KREG_D, 1>(p, s, bar, 0, r, nullptr, nullptr, nullptr, p.d, p.Kpd, resid);
}

// Copies one matrix into the tile order of its kind: tile T of the packed stream is
// (strip, k-tile) = desc[T]; lane l holds row l%16, columns 8*(l/16)..+7 of that tile.
__global__ void repack_kernel(const uint16_t* W, int K, int kind, int m, int row0, const uint32_t* desc, uint4* out) {
    const size_t tile = blockIdx.x;
    const int lane = threadIdx.x;
    const uint32_t dsc = desc[tile];
    const int strip = dsc >> 12, kt = dsc & 4095, r = lane & 15;
    size_t row = (size_t)(row0 + strip * 16 + r), col = (size_t)kt * 32 + (lane >> 4) * 8;
    if (kind == K_D) row = (size_t)((r < 8 ? 0 : m) + strip * 8 + (r & 7));
    if (kind == K_WD) {  // strip = block * (d/16) + s of the [d, 3d] matrix, K = 3d, row0 carries d
        const int per = row0 / 16, blk = strip / per;
        row = (size_t)((strip - blk * per) * 16 + r);
        col += (size_t)blk * row0;
    }
    out[tile * 64 + lane] = *reinterpret_cast<const uint4*>(W + row * K + col);
}

// ------------------------------------------------------------------------- host: plan

struct KindPlan {
    int nstrips, KT, TPS, maxS, rounds;
    int ksplit;          // workgroups that share one strip, each with 1/ksplit of K (W2 only; else 1)
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
    unsigned epoch;     // grid barriers completed by all launches so far
    unsigned launches;
    bool err_word_ready;   // the error word (shared with the kernel laid out on the XCDs) has been cleared
};

namespace {

bool shape_ok(const hawk_ctx* c) {
    if (c->cfg.dtype != HAWK_BF16) return false;
    if (c->hd != 64) return false;
    if (c->d % 128 || c->m % 128 || c->Vs % 16 || (3 * c->d) % 128) return false;
    if (c->d / 128 > kTMax || c->m / 128 > kTMax) return false;
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
    // The draft projection W_d [d, 3d] is planned as three [d, d] blocks (previous head output,
    // left neighbour, upper neighbour): 3 d/16 strips whose partial outputs the consumer adds.
    const int nstrips[K_NKIND] = {3 * d / 16, d / 16, 2 * m / 16, d / 16, c->Vs / 16, 3 * d / 16};
    const int KT[K_NKIND] = {d / 32, d / 32, d / 32, m / 32, d / 32, d / 32};
    for (int k = 0; k < K_NKIND; ++k) {
        KindPlan& kp = P->kind[k];
        kp.nstrips = nstrips[k]; kp.KT = KT[k];
        kp.ksplit = 1;
        if (k == K_E) {  // W2 has few, long strips: as many workgroups per strip as divide its K evenly
            for (int f = kNWG / nstrips[k]; f > 1; --f)
                if (KT[k] % (4 * f) == 0) { kp.ksplit = f; break; }
        }
        kp.TPS = KT[k] / (4 * kp.ksplit);
        kp.maxS = std::min(kMaxStrips, kTMax / kp.TPS);
        kp.tiles = (size_t)nstrips[k] * KT[k];
        kp.rounds = k <= K_E ? 1 : (nstrips[k] + kNWG * kp.maxS - 1) / (kNWG * kp.maxS);
        if (k <= K_E && nstrips[k] > kNWG * kp.maxS) { P->ok = false; return; }
    }
    std::vector<std::vector<int>> assign[K_NKIND];  // [kind][round][wg] -> strips
    for (int k = 0; k < K_NKIND; ++k) assign[k].assign((size_t)P->kind[k].rounds * kNWG, {});
    // Wo and W2: strip s of both belongs to workgroup s, which keeps that strip of the residual
    // stream in registers for the whole launch (workgroup s runs on XCD s % 8).
    if (nstrips[K_C] > kNWG || nstrips[K_E] != nstrips[K_C]) { P->ok = false; return; }
    std::vector<long> load(kNWG, 0);
    const int fE = P->kind[K_E].ksplit;
    for (int s = 0; s < nstrips[K_C]; ++s) {
        assign[K_C][s].push_back(s);
        load[s] += P->kind[K_C].TPS;
    }
    // W2: part j of strip s (K range j / fE) goes to workgroup j * strips + s; part 0 - the owner of
    // the residual strip - adds the other parts' partial sums (entry = part * strips + strip)
    for (int j = 0; j < fE; ++j)
        for (int s = 0; s < nstrips[K_E]; ++s) {
            assign[K_E][(size_t)j * nstrips[K_E] + s].push_back(j * nstrips[K_E] + s);
            load[(size_t)j * nstrips[K_E] + s] += P->kind[K_E].TPS;
        }
    // QKV and W1|W3: as few strips per workgroup as the count allows, the extra ones to the
    // workgroups that stream least per layer.
    const int order[2] = {K_D, K_A};
    for (int oi = 0; oi < 2; ++oi) {
        const int k = order[oi];
        const int cap = (nstrips[k] + kNWG - 1) / kNWG;
        if (cap > P->kind[k].maxS) { P->ok = false; return; }
        for (int s = 0; s < nstrips[k]; ++s) {
            int best = -1;
            for (int g = 0; g < kNWG; ++g)
                if ((int)assign[k][g].size() < cap && (best < 0 || load[g] < load[best])) best = g;
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
                int kt0 = 0;
                if (k == K_E && ns) {  // (strip, part) in the first two fields
                    s3[0] = st[0] % kp.nstrips; s3[1] = st[0] / kp.nstrips;
                    kt0 = s3[1] * (kp.KT / kp.ksplit);
                }
                P->tab.push_back((int32_t)tile);
                P->tab.push_back(ns);
                P->tab.push_back((int32_t)((unsigned)s3[0] | ((unsigned)s3[1] << 16)));
                P->tab.push_back(s3[2]);
                for (int wv = 0; wv < kCW; ++wv)
                    for (int t = 0; t < ns * kp.TPS; ++t) {
                        P->desc.push_back(((uint32_t)(k == K_E ? s3[0] : st[t / kp.TPS]) << 12) |
                                          (uint32_t)(kt0 + wv * kp.TPS + t % kp.TPS));
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

// Regions of an exchange slot, in floats: split planes are uint16 [16][K + 8] (hi, lo), sums of
// squares [d / 16][16], queries [16][d], attention chunk partials.  Returns the slot size.
size_t slot_layout(const hawk_ctx* c, SP* p) {
    const size_t d = c->d, m = c->m, pd = 8 * (d + 8), pm = 8 * (m + 8);
    size_t at = 0;
    auto take = [&](size_t n) { size_t a = at; at += (n + 63) & ~(size_t)63; return a; };
    const size_t xh = take(pd), xl = take(pd), ssx = take(d), q = take(16 * d), oh = take(pd), ol = take(pd);
    const size_t x2h = take(pd), x2l = take(pd), ss2 = take(d), hh = take(pm), hl = take(pm);
    const size_t pp = take((size_t)kNWG * 8 * kPS);
    const size_t ep = take((size_t)kNWG * 256);   // W2 partial strips: [strip * (parts - 1) + part - 1][64 lanes][4]
    if (p) {
        p->o_ep = ep;
        p->o_xh = xh; p->o_xl = xl; p->o_ssx = ssx; p->o_q = q; p->o_oh = oh; p->o_ol = ol;
        p->o_x2h = x2h; p->o_x2l = x2l; p->o_ss2 = ss2; p->o_hh = hh; p->o_hl = hl; p->o_p = pp;
    }
    return at;
}

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
    // one exchange slot per layer (+1), kRing arenas
    o->slot_bytes = up256(slot_layout(c, nullptr) * 4);
    o->arena = take(o->slot_bytes * (L + 1) * kRing);
    o->bar = take((size_t)(kGroups + 1 + kReplicas) * 4096);
    o->err = take(256);
    o->dbg = take((4 * 4096 * 8 + 2 * 256 * kNWG) * 8);
    o->rope = take((size_t)c->Tmax * (c->hd / 2) * 8);
    return p - base;
}

StreamPlan* stream_create(hawk_ctx* c) {
    StreamPlan* P = new StreamPlan();
    build_plan(c, P);
    P->epoch = 0;
    P->launches = 0;
    P->err_word_ready = false;
    if (!P->ok) return P;
    {   // the grid barrier needs all kNWG workgroups resident at once: one per compute unit
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < kNWG) {
            P->ok = false;
            return P;
        }
    }
    const StreamOffsets& o = c->soff;
    std::vector<float> rope((size_t)c->Tmax * (c->hd / 2) * 2);
    for (int pos = 0; pos < c->Tmax; ++pos)
        for (int j = 0; j < c->hd / 2; ++j) {
            const double ang = (double)pos * pow((double)c->cfg.rope_theta, -2.0 * j / (double)c->hd);
            rope[((size_t)pos * (c->hd / 2) + j) * 2] = (float)cos(ang);
            rope[((size_t)pos * (c->hd / 2) + j) * 2 + 1] = (float)sin(ang);
        }
    // tables, rotary table, zeroed barrier memory - on the context's stream, every return code checked: a
    // plan whose tables did not reach the device must never be launched
    bool good = true;
    auto up = [&](size_t off, const void* src, size_t bytes) {
        good = good && hipMemcpyAsync(c->ws + off, src, bytes, hipMemcpyHostToDevice, c->stream) == hipSuccess;
    };
    auto fill = [&](size_t off, int value, size_t bytes) {
        good = good && hipMemsetAsync(c->ws + off, value, bytes, c->stream) == hipSuccess;
    };
    up(o.tab, P->tab.data(), P->tab.size() * 4);
    up(o.desc, P->desc.data(), P->desc.size() * 4);
    fill(o.bar, 0, (size_t)(kGroups + 1 + kReplicas) * 4096);
    // every word of the exchange arenas starts as the "not written yet" pattern the W2 stage polls for
    fill(o.arena, 0xFF, o.slot_bytes * (size_t)(c->L + 1) * kRing);
    fill(o.err, 0, 256);
    up(o.rope, rope.data(), rope.size() * 4);
    good = good && hipStreamSynchronize(c->stream) == hipSuccess;   // the sources are locals and plan members
    if (!good) {
        (void)hipGetLastError();
        P->ok = false;   // the context falls back to one kernel per operation
    }
    P->err_word_ready = good;
    if (good) { c->err_off = o.err; c->rope_off = o.rope; c->err_ready = 1; }
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

// How the attention stage is cut into jobs for steps of RS rows per sequence: one job per
// (sequence, head, row), times NC chunks of the cached positions while the jobs of the heads
// that share an XCD still fit its 32 workgroups (with one chunk the job emits finished rows).
struct AttnCut { int NRG, RPJ, NC; bool ok; };
static AttnCut attn_cut(const hawk_ctx* c, int RS) {
    const int heads_per_xcd = (c->S * c->H + kXcd - 1) / kXcd;
    AttnCut a;
    a.NRG = RS;
    a.RPJ = 1;
    a.ok = heads_per_xcd * RS <= kPerXcd;
    a.NC = a.ok ? std::min(kNCMax, kPerXcd / (heads_per_xcd * RS)) : 1;
    return a;
}

// Elements between the hi and the lo plane rows in LDS: the longest stage input a workgroup
// stages (d, or its share of m in the W2 stage), padded.
static size_t act_stride(const hawk_ctx* c) {
    const int f = c->plan ? c->plan->kind[K_E].ksplit : 1;
    return (size_t)std::max(c->d, c->m / f) + 8;
}

// LDS of one workgroup: activation hi/lo planes (or, during attention, the per-wave partials),
// K-quarter partial strips, row scales, scaled queries, IO join word.
static size_t stream_lds_bytes(const hawk_ctx* c, int MR) {
    const size_t act = std::max((size_t)MR * act_stride(c) * 4, (size_t)kCW * 6 * kPS * 4);
    return act + (size_t)(kCW * kMaxStrips * 256 + 16 + 6 * 64 + 16) * 4;
}

bool stream_ok(const hawk_ctx* c, int k) {
    if (!c->plan || !c->plan->ok || c->path < 1) return false;
    const int MR = c->S * (k + 1);
    if (MR > 16 || k + 1 > 6) return false;
    if (!attn_cut(c, k + 1).ok) return false;
    return stream_lds_bytes(c, MR) <= 150 * 1024;
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
    run(c->w.W_d, 3 * c->d, K_WD, P->wd_base, c->d);
    if (hipGetLastError() != hipSuccess) return -1;
    return hipStreamSynchronize(c->stream) == hipSuccess ? 0 : -1;
}

// Kernel parameters common to the target pass and the draft head for a launch over MR rows.
static void fill_params(hawk_ctx* c, SP& p, int MR) {
    StreamPlan* P = c->plan;
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
    p.blob = wsp<uint16_t>(c, c->off.blob);
    p.g1_off = c->w.g1[0]; p.g2_off = c->w.g2[0];
    p.layer_bytes = c->L > 1 ? c->w.g1[1] - c->w.g1[0] : 0;
    p.gf_off = c->w.g_f;
    p.rope = wsp<float2>(c, o.rope);
    p.Kc = wsp<_Float16>(c, c->off.kc); p.Vc = wsp<_Float16>(c, c->off.vc);
    p.X = wsp<float>(c, c->off.x);
    p.arena = wsp<float>(c, o.arena + (size_t)(P->launches % kRing) * o.slot_bytes * (c->L + 1));
    p.slot_floats = o.slot_bytes / 4;
    (void)slot_layout(c, &p);
    p.dbg = c->stream_dbg ? wsp<u64>(c, o.dbg) : nullptr;
    p.bar = wsp<unsigned>(c, o.bar); p.err = wsp<unsigned>(c, o.err);
    p.n = wsp<int32_t>(c, c->off.n); p.k_eff = wsp<int32_t>(c, c->off.k_eff);
    p.epoch0 = P->epoch;
    p.L = c->L; p.d = c->d; p.H = c->H; p.m = c->m; p.Vs = c->Vs; p.S = c->S; p.B = c->B; p.C = c->C;
    p.MR = MR;
    p.Smax = c->Smax; p.Tmax = c->Tmax; p.Kpd = c->d + 8; p.Kpm = c->m + 8;
    p.esplit = P->kind[K_E].ksplit; p.KpE = c->m / p.esplit + 8;
    p.eps = c->cfg.rms_eps;
    p.act_bytes = (int32_t)std::max((size_t)p.MR * act_stride(c) * 4, (size_t)kCW * 6 * kPS * 4);
}

static int launch_persistent(hawk_ctx* c, const void* kern, SP& p, unsigned barriers) {
    StreamPlan* P = c->plan;
    const size_t lds = stream_lds_bytes(c, p.MR);
    if (hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess) return -1;
    void* args[] = {&p};
    // An ordinary launch: every workgroup gets a compute unit of its own because the grid is
    // exactly the number of units, one workgroup fills a unit's LDS, and the stream's previous
    // kernel has drained (checked once in stream_create; the barrier's waits are bounded in any
    // case).  A cooperative launch costs ~11 us of idle queue on either side on this runtime.
    if (hipLaunchKernel(kern, dim3(kNWG), dim3(kThreads), args, lds, c->stream) != hipSuccess) return -1;
    P->epoch += barriers;
    P->launches += 1;
    return 0;
}

// Enqueues the target pass over the step rows; X (c->off.x) must hold the embedded rows.
// Returns 0, or -1 if the launch failed.
int launch_verify_stream(hawk_ctx* c, int k) {
    SP p;
    fill_params(c, p, c->S * (k + 1));
    p.logit_s = wsp<float>(c, c->off.logit_s);
    p.RS = k + 1;
    const AttnCut cut = attn_cut(c, k + 1);
    p.NC = cut.NC; p.NRG = cut.NRG; p.RPJ = cut.RPJ;
    const void* kern = c->d == 1280 ? reinterpret_cast<const void*>(verify_stream_kernel<10, 9, 5, 6>)
                                    : reinterpret_cast<const void*>(verify_stream_kernel<6, 4, 3, 6>);
    // prologue + five stages per layer; nothing follows the output projection
    return launch_persistent(c, kern, p, 1u + 5u * (unsigned)c->L);
}

// Tree rows on the streaming path: the nodes of one candidate tree per sequence, at most 16 rows in
// all, two rows per attention job (their jobs must fit the workgroups of an XCD).
bool stream_tree_ok(const hawk_ctx* c, int n_nodes) {
    if (!c->plan || !c->plan->ok || c->path < 1) return false;
    const int MR = c->S * n_nodes;
    if (MR > 16 || n_nodes < 1) return false;
    const int heads_per_xcd = (c->S * c->H + kXcd - 1) / kXcd;
    if (heads_per_xcd * ((n_nodes + 1) / 2) > kPerXcd) return false;
    return stream_lds_bytes(c, MR) <= 150 * 1024;
}

int launch_verify_stream_tree(hawk_ctx* c, int n_nodes, const int32_t* tree_depth, const unsigned long long* tree_anc) {
    SP p;
    fill_params(c, p, c->S * n_nodes);
    p.logit_s = wsp<float>(c, c->off.logit_s);
    p.RS = n_nodes;
    // one row per attention job while the jobs of the heads that share an XCD fit its workgroups, else two
    const int heads_per_xcd = (c->S * c->H + kXcd - 1) / kXcd;
    const bool single = heads_per_xcd * n_nodes <= kPerXcd;
    p.NC = 1; p.RPJ = single ? 1 : 2; p.NRG = single ? n_nodes : (n_nodes + 1) / 2;
    p.tdepth = tree_depth;
    p.tanc = reinterpret_cast<const u64*>(tree_anc);
    const void* kern =
        c->d == 1280 ? (single ? reinterpret_cast<const void*>(verify_stream_kernel<10, 9, 5, 6, true, 1>)
                               : reinterpret_cast<const void*>(verify_stream_kernel<10, 9, 5, 6, true, 2>))
                     : (single ? reinterpret_cast<const void*>(verify_stream_kernel<6, 4, 3, 6, true, 1>)
                               : reinterpret_cast<const void*>(verify_stream_kernel<6, 4, 3, 6, true, 2>));
    return launch_persistent(c, kern, p, 1u + 5u * (unsigned)c->L);
}

// Can draft micro-steps run on the streaming path?
bool stream_draft_ok(const hawk_ctx* c) {
    if (!c->plan || !c->plan->ok || c->path < 1) return false;
    return c->S <= 16 && stream_lds_bytes(c, c->S) <= 150 * 1024 && c->plan->kind[K_WD].rounds == 1;
}

// Enqueues draft micro-step i (1-based) up to its logits: the head's hidden state goes to
// off_out ([S][d] fp32), reading the previous one from off_prev; logits to dlogit_s.
int launch_draft_stream(hawk_ctx* c, int i, size_t off_prev, size_t off_out) {
    SP p;
    fill_params(c, p, c->S);
    p.logit_s = wsp<float>(c, c->off.dlogit_s);
    p.RS = 1; p.NC = 1; p.NRG = 1; p.RPJ = 1;
    p.prev = wsp<float>(c, off_prev);
    p.gout = wsp<float>(c, off_out);
    p.dpart = p.arena + p.o_p;   // slot 0's attention-partial region: 3 * 16 * d floats fit
    p.grid = wsp<int32_t>(c, c->off.grid);
    p.draft = wsp<int32_t>(c, c->off.draft);
    p.E_off = c->w.E;
    p.step_i = i; p.N = c->N; p.IW = c->gw; p.kstride = c->kmax + 1;
    const void* kern = c->d == 1280 ? reinterpret_cast<const void*>(draft_stream_kernel<10, 5, 6>)
                                    : reinterpret_cast<const void*>(draft_stream_kernel<6, 3, 6>);
    return launch_persistent(c, kern, p, 1u);
}

// The persistent kernels' error word exists and has been cleared (its region is part of the workspace
// whenever the shape has a streaming plan; the kernel laid out on the XCDs shares it).
bool stream_has_err_word(const hawk_ctx* c) { return c->err_ready != 0; }

// 1 if a wait of the persistent kernels ever timed out (the result of that step is invalid).
int stream_error(hawk_ctx* c) {
    if (!stream_has_err_word(c)) return 0;
    unsigned e = 0;
    if (hipMemcpyAsync(&e, c->ws + c->err_off, 4, hipMemcpyDeviceToHost, c->stream) != hipSuccess) return 1;
    if (hipStreamSynchronize(c->stream) != hipSuccess) return 1;
    return e != 0;
}

}  // namespace hawk
