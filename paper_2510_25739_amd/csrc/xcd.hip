// Target pass over the k+1 rows of a step as ONE persistent kernel laid out on the chip's eight XCDs
// (32 compute units and one L2 each): the dependent chain of a layer runs on flags and data that
// cross between XCDs once per matrix product and otherwise stay inside one XCD's L2.
//
// Measured on MI355X (256 workgroups, one per unit): a store that goes through to memory is seen by a
// polling workgroup of another XCD after ~0.55 us; inside an XCD an ordinary store (it stays in that
// XCD's L2) is seen by a device-scope load of another unit after ~0.22 us; a grid barrier plus the
// fetch of a fresh 32 KB input by every workgroup costs ~4.0 us, which bounds a kernel that exchanges
// whole activation vectors between all workgroups five times per layer at ~6 us per stage.
//
// Hence, per matrix product y = W x:
//   - XCD c owns a K-slice of x (an eighth of the columns; for the attention output the columns of the
//     heads it owns; for the MLP's hidden vector an eighth of its k-tiles) and keeps it in a buffer only
//     its own units read: consumers fetch an eighth of the vector, from their own L2;
//   - workgroup (c, j) streams the weights of its output strips x that K-slice (bf16 tiles straight into
//     registers as MFMA A operands, one wave per strip group, no cross-wave reduction) and writes the
//     partial sums to memory as fp32 values whose lowest mantissa bit carries the parity of the number of
//     times the word has been written (a reader knows a word is of this stage without any barrier, and
//     nothing has to be re-armed);
//   - the strip's owner - an IO wave on the XCD that owns those output columns as its K-slice of the
//     NEXT product - polls the eight partials, adds them in fixed order, applies the epilogue (norm
//     scale, rotary embedding, residual, SwiGLU), stores the result into its XCD's buffer with ordinary
//     stores and raises a flag word there; the XCD's units poll those flag words (one L2 line).
// Attention for a head runs on the XCD that owns the head: queries, new keys/values and the output
// rows never leave that XCD.  A product that follows a norm needs every row's sum of squares over the
// whole vector: each XCD sums its slice while staging it and sends that share along with its partial
// sums (one tagged word per wave and row), so the owner has norm scale and dot products from the same
// poll.  No grid barrier anywhere; every wait is a bounded poll that ends in an error code.
//
// In the loaded kernel the latencies are two to three times the idle ones (a partial sum is in its
// owner's registers 1.3 - 2.7 us after its store was issued, a local flag is seen after ~0.4 us, the
// staging copy takes ~0.55 us), which is what bounds a stage at 4.4 - 5.5 us at the XL shape (see the
// stage table that hawk_phase_trace gives); the weight stream itself accounts for ~5 % of that kernel's
// time.  Two forms of the compute side: verify_xcd_kernel keeps a layer's tiles in registers, requested
// a fifth of a layer per stage (d_model 768 / 1280); verify_xcd_stream_kernel streams them through two
// register buffers (d_model 4096, where the stream is two thirds of the time).  The IO side is shared.
#include <math.h>
#include <stdlib.h>
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

constexpr int kCW = 4, kNIO = 4;                 // compute / IO waves per workgroup
constexpr int kThreads = (kCW + kNIO) * 64, kIOThreads = kNIO * 64;
constexpr int kXcd = 8, kPer = kNWG / kXcd;      // workgroup i runs on XCD i % 8 (checked by every workgroup)
constexpr unsigned kSpinLimit = 1u << 20;
constexpr int kNIT = 4;                          // cache positions per lane group and register buffer
constexpr int kPaceGap = 0, kPaceTiles = 6;   // weight requests go out six tiles per wave at a time (see issue_paced)
constexpr int kRing = 2;                         // partial-sum areas and XCD buffers alternate between layers
constexpr int kMaxJobs = 128;                    // flag words of one XCD and stage that others wait for (one per IO wave with a job)

enum XKind { X_A = 0, X_C, X_D, X_E, X_LM, X_NK };   // QKV, Wo, W1|W3, W2, output projection
enum XFlag { F_A = 0, F_B, F_C, F_D, F_E, F_NF };    // who raised a flag: reduce of A, attention, reduce of C, D, E

struct XP {
    const uint4* wpack;
    const uint4* zero_tile;     // 1 KB of zeros: what absent strips / k-tiles of a wave's job read
    u64 layer_tiles;            // tiles of one layer
    u64 xbase[X_NK][kXcd];      // first tile of (kind, XCD) inside a layer (output projection: after all layers)
    int32_t KT[X_NK][kXcd];     // k-tiles of the XCD's slice of the kind's input
    int32_t nstrips[X_NK];
    int32_t hd0[kXcd + 1];      // heads of XCD c: hd0[c] .. hd0[c + 1] - 1
    int32_t ke0[kXcd + 1];      // k-tiles of the MLP's hidden vector of XCD c
    const int16_t* gtab;        // [kind][32][kCW][2]: first strip and strip count of (unit j, compute wave w)
    const int16_t* ptab;        // [poff[kind] + strip]: producer of the strip, (unit * kCW + wave) * 2 + round
    int poff[X_NK];
    const int16_t* rtab;        // [kind][8][32][kNIO][3]: strip (-1: none), flag slot, second strip (-1: none) of (XCD, unit, IO wave)
    const int16_t* atab;        // [8][32][4]: sequence, head, row group (-1: none), flag slot
    int32_t njobs[F_NF][kXcd];  // flag slots a consumer of that stage waits for
    u64* part[X_NK];            // partial sums: [ring][8 source XCDs][strip][16 rows][16 features] fp32, parity in the lowest bit
    u64* pss[X_NK];             // per-XCD sums of squares that ride along (products after a norm): [ring][8][unit][wave][round][16 rows] {value, tag}
    uint8_t* xbuf;              // per-XCD buffers: [8][ring][xcd_bytes]
    u64 xcd_bytes, o_a, o_q, o_kv, o_o, o_x2, o_h, o_ss;   // regions of one XCD buffer (bytes)
    unsigned* lflag;            // [8][F_NF][kMaxJobs]
    const uint16_t* blob;
    u64 g1_off, g2_off, layer_bytes, gf_off;
    const float2* rope;
    _Float16* Kc;
    _Float16* Vc;
    float* X;                   // embedded rows in, final hidden rows out ([MR][d] fp32)
    float* logit_s;
    unsigned* err;
    const int32_t* n;
    const int32_t* k_eff;
    const int32_t* tdepth;      // rows of a candidate tree (null: a chain): depth of node r, and bit a of tanc[r] set iff node a
    const u64* tanc;            //   is an ancestor of node r; node r sits at the root's position + depth, in cache entry root + r
    int32_t L, d, H, m, Vs, S, B, C, RS, MR, RPJ, Smax, Tmax;
    int32_t hd;                 // head dimension (64 or 128)
    float qscale;               // 1 / sqrt(hd)
    int32_t KpA, KpO, KpH;      // row strides (elements) of the split planes: d / 8 + 8, widest head group + 8, widest hidden slice + 8
    int32_t lm_rounds;
    float eps;
};

// ------------------------------------------------------------------------- device helpers

__device__ __forceinline__ unsigned xcc_id() {
    unsigned v;
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(v));
    return v & 0xFu;
}
// A 64-bit value that is the same in every lane, moved to scalar registers.  (The builtin returns int: each
// half goes through unsigned, or a low half with its top bit set would spill ones over the high half.)
__device__ __forceinline__ unsigned long long uniform64(unsigned long long v) {
    const unsigned lo = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)v);
    const unsigned hi = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)(v >> 32));
    return ((unsigned long long)hi << 32) | (unsigned long long)lo;
}
__device__ __forceinline__ void compiler_fence() { __atomic_signal_fence(__ATOMIC_SEQ_CST); }
// A pointer the compiler must treat as new: addresses derived from it are computed where they are used
// instead of once before the layer loop (dozens of 64-bit addresses kept alive across the whole kernel).
template <typename T>
__device__ __forceinline__ T* fresh(T* ptr) {
    asm volatile("" : "+v"(ptr));
    return ptr;
}

// Loads that must see what another unit of the same XCD stored (they skip the unit's own L1 and are
// served by the XCD's L2), or what another XCD wrote through to memory: device scope.  The 16-byte forms
// go through a buffer resource (32-bit byte offsets from a wave-uniform base), which the compiler tracks
// like any other load.
typedef __amdgpu_buffer_rsrc_t rsrc_t;
constexpr int kDevScope = 16;   // cache-policy bit of device scope in the buffer instructions
constexpr int kNonTemporal = 2; // ... of a streaming access (no reuse expected)
__device__ __forceinline__ rsrc_t make_rsrc(const void* base) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, 0x7FFFFFFF, 0x00020000);
}
__device__ __forceinline__ v4u ld_16(rsrc_t r, unsigned byte_off) {
    return __builtin_amdgcn_raw_buffer_load_b128(r, byte_off, 0, kDevScope);
}
__device__ __forceinline__ void st_16(rsrc_t r, unsigned byte_off, v4u v) {   // goes through to memory
    __builtin_amdgcn_raw_buffer_store_b128(v, r, byte_off, 0, kDevScope);
}
__device__ __forceinline__ u64 ld_u64(const void* p) {
    return __hip_atomic_load(reinterpret_cast<const u64*>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned ld_u32(const void* p) {
    return __hip_atomic_load(reinterpret_cast<const unsigned*>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// Stores that go through to memory (sums of squares: read by other XCDs).
__device__ __forceinline__ void st_tagged(u64* p, float v, unsigned tag) {
    __hip_atomic_store(p, (u64)__float_as_uint(v) | ((u64)tag << 32), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

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
__device__ __forceinline__ float lane_xor8(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x128, 0xF, 0xF, true));
}

__device__ __forceinline__ unsigned bf16_rne(float f) {
    unsigned u = __float_as_uint(f);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}
__device__ __forceinline__ float bf16_f32(unsigned b) { return __uint_as_float(b << 16); }

// Four consecutive elements of a split vector (bf16 hi and lo halves), ordinary stores: the XCD's buffer.
__device__ __forceinline__ void put_split4(uint16_t* hi, uint16_t* lo, f32x4 v) {
    const unsigned h0 = bf16_rne(v[0]), h1 = bf16_rne(v[1]), h2 = bf16_rne(v[2]), h3 = bf16_rne(v[3]);
    const unsigned l0 = bf16_rne(v[0] - bf16_f32(h0)), l1 = bf16_rne(v[1] - bf16_f32(h1));
    const unsigned l2 = bf16_rne(v[2] - bf16_f32(h2)), l3 = bf16_rne(v[3] - bf16_f32(h3));
    *reinterpret_cast<uint2*>(hi) = make_uint2(h0 | (h1 << 16), h2 | (h3 << 16));
    *reinterpret_cast<uint2*>(lo) = make_uint2(l0 | (l1 << 16), l2 | (l3 << 16));
}
__device__ __forceinline__ f32x4 times_gain(f32x4 x, uint2 g) {
    return (f32x4){x[0] * bf16_f32(g.x & 0xFFFFu), x[1] * bf16_f32(g.x >> 16), x[2] * bf16_f32(g.y & 0xFFFFu),
                   x[3] * bf16_f32(g.y >> 16)};
}

// State of one wave: where it sits, the stage counter, whether a wait has given up.
struct Ctx {
    unsigned x, j;        // XCD and unit of the workgroup
    unsigned epoch0;      // tags of this launch start behind it
    unsigned par;         // partial sums: bit r of the low / high half = parity of the writes so far to row r's words of the
                          //   even / odd layers' areas; bits 0..15 of par_lm the same for the output projection's
    unsigned par_lm;
    bool dead;
    unsigned* err;
    u64* dbg;             // time stamps of two workgroups (null: off)
};

// Tag of (layer, stage); the prologue counts as stage E of layer -1.
__device__ __forceinline__ unsigned tag_of(const Ctx& c, int layer, int flag) {
    return c.epoch0 + 1u + 5u * (unsigned)(layer + 1) + (unsigned)flag;
}

// Partial sums carry no tag word: the lowest mantissa bit of every value is the parity of the number of
// times its word has been written (the word is rewritten every second layer, by every launch, for the rows
// in flight; the host keeps the parities per row between launches).  A reader that finds the expected
// parity in all four values of a 16-byte word has the stage's values; it clears the bit before use, so the
// sums do not depend on it.  Half the bytes of {value, tag} pairs cross between the XCDs.
__device__ __forceinline__ unsigned parity_bit(const Ctx& c, int kind, int layer, int row) {
    const unsigned base = kind == X_LM ? c.par_lm >> row : c.par >> (16 * (layer & 1) + row);
    return (base ^ (kind == X_LM ? 0u : (unsigned)(layer >> 1)) ^ 1u) & 1u;
}

__device__ __forceinline__ void give_up(Ctx& c) {
    c.dead = true;
    __hip_atomic_store(c.err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Waits until the first `n` flag words of this XCD's stage `flag` have reached `tag` (whole wave).
__device__ __forceinline__ void wait_flags(const XP& p, Ctx& c, int flag, int n, unsigned tag) {
    if (c.dead) return;
    const unsigned l = threadIdx.x & 63u;
    const unsigned* f = p.lflag + ((size_t)c.x * F_NF + flag) * kMaxJobs;
    const unsigned i0 = l < (unsigned)n ? l : 0u, i1 = l + 64u < (unsigned)n ? l + 64u : 0u;   // a lane looks at flags l and l + 64
    for (unsigned spins = 0; spins < kSpinLimit; ++spins) {
        const unsigned v = ld_u32(f + i0);
        const unsigned w = n > 64 ? ld_u32(f + i1) : v;
        if (__all((int)(v - tag) >= 0 && (int)(w - tag) >= 0)) { compiler_fence(); return; }
        if ((spins & 255u) == 255u && ld_u32(c.err) != 0u) break;
    }
    give_up(c);
}

// After the wave's ordinary stores into the XCD's buffer: they are in the L2 once acknowledged, then
// the flag word goes up.
__device__ __forceinline__ void raise_flag(const XP& p, const Ctx& c, int flag, int slot, unsigned tag) {
    __builtin_amdgcn_s_waitcnt(0);
    if ((threadIdx.x & 63u) == 0u)
        __hip_atomic_store(p.lflag + ((size_t)c.x * F_NF + flag) * kMaxJobs + slot, tag, __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_WORKGROUP);
}

__device__ __forceinline__ uint8_t* xcd_buf(const XP& p, unsigned x, int ring) {
    return p.xbuf + ((size_t)x * kRing + ring) * p.xcd_bytes;
}

__device__ __forceinline__ void stamp(const Ctx& c, unsigned stage, int what) {
    if (c.dbg && (threadIdx.x & 63) == 0 && (blockIdx.x == 0 || blockIdx.x == 248) && stage < 512u)
        c.dbg[((size_t)(blockIdx.x ? 1 : 0) * 512 + stage) * 16 + what + ((threadIdx.x >> 6) >= kCW ? 8 : 0)] =
            __builtin_amdgcn_s_memrealtime();
}

struct RowPos { int seq, r, pos, slot; bool valid; };   // pos: rotary position; slot: cache entry
__device__ __forceinline__ RowPos row_pos(const XP& p, int c) {
    RowPos o;
    o.seq = c / p.RS;
    o.r = c - o.seq * p.RS;
    const int b = o.seq % p.B;
    o.valid = o.r <= p.k_eff[b];
    o.slot = o.valid ? p.C + p.n[b] - 1 + o.r : 0;
    o.pos = (o.valid && p.tdepth) ? p.C + p.n[b] - 1 + p.tdepth[o.r] : o.slot;
    return o;
}

// ------------------------------------------------------------------------- matrix products

// A compute wave's share of one kind of product, read from the tables once at kernel start (a table
// load behind a workgroup barrier would sit on every stage's critical path).
struct GJob {
    int s0, ns, KT;   // first strip, strips, k-tiles of the XCD's slice
    u64 tile0;        // first tile inside a layer (output projection: in the stream)
};
__device__ __forceinline__ GJob load_gjob(const XP& p, int kind, const Ctx& c, int wave) {
    const int16_t* g = p.gtab + (((size_t)kind * kPer + c.j) * kCW + wave) * 2;
    GJob j;
    j.s0 = g[0]; j.ns = g[1]; j.KT = p.KT[kind][c.x];
    j.tile0 = p.xbase[kind][c.x] + (u64)j.s0 * j.KT;
    return j;
}

// Issues the loads of a wave's tiles of one stage: strips x the XCD's k-tiles, in that order in the
// packed stream.  Straight-line code: absent strips / k-tiles read one shared tile of zeros (a cache
// hit), so that the number of requests is fixed and the wait before the products can be for exactly
// this stage's tiles - not for the tiles of later stages requested behind them.
template <int NSW, int KTM, int T0 = 0, int T1 = NSW * KTM>
__device__ __forceinline__ void issue_tiles(const XP& p, const GJob& g, u64 layer_base, int lane, v4u (&w)[NSW * KTM],
                                            int round = 0) {
    const int ns = min(max(g.ns - round * NSW, 0), NSW), KT = g.KT;
    const v4u* src = reinterpret_cast<const v4u*>(p.wpack + (layer_base + g.tile0 + (u64)round * NSW * KT) * 64 + lane);
    const v4u* zero = reinterpret_cast<const v4u*>(p.zero_tile) + lane;
#pragma unroll
    for (int t = T0; t < T1; ++t) {   // (a sub-range of the wave's tiles: a request can be spread over several stages)
        const int si = t / KTM, kt = t % KTM;
        const bool on = si < ns && kt < KT;
        w[t] = __builtin_nontemporal_load(on ? src + (size_t)(si * KT + kt) * 64 : zero);
    }
}
// The same in parts of at most CH tiles, each waited for before the next is requested: what another wave
// of the unit asks for in between waits for one part, not for the whole request.
template <int NSW, int KTM, int T0, int T1, int CH>
__device__ __forceinline__ void issue_paced(const XP& p, const GJob& g, u64 layer_base, int lane, v4u (&w)[NSW * KTM]) {
    if constexpr (T0 < T1) {
        constexpr int TE = T0 + CH < T1 ? T0 + CH : T1;
        issue_tiles<NSW, KTM, T0, TE>(p, g, layer_base, lane, w);
        if (kPaceGap >= 0) {
            __builtin_amdgcn_s_waitcnt(0x0f70);   // vmcnt(0)
            if (kPaceGap > 0) __builtin_amdgcn_s_sleep(kPaceGap);
        }
        issue_paced<NSW, KTM, TE, T1, CH>(p, g, layer_base, lane, w);
    }
}

// The wave's products of a stage from the staged K-slice (LDS planes [16][Kp]) and the partial sums
// out as tagged words: part[ring][XCD][strip][row][quad][4].  No branches up to the stores (see above).
template <int NSW, int KTM>
__device__ __forceinline__ void mfma_store(const XP& p, int kind, const GJob& g, const Ctx& c, int lane, const v4u (&w)[NSW * KTM],
                                           const uint16_t* act_hi, const uint16_t* act_lo, const float* ssrow, int Kp, int ring,
                                           unsigned tag, unsigned pbit, int round = 0, unsigned dbg_stage = 0) {
    const int s0 = g.s0 + round * NSW, ns = min(max(g.ns - round * NSW, 0), NSW);
    const int col = lane & 15, kg = lane >> 4;
    const size_t at = (size_t)(col < p.MR ? col : 0) * Kp + kg * 8;
    if (ssrow && kg == 0 && col < p.MR && ns > 0)   // the product follows a norm: this XCD's share of the row's sum of squares
                                                    // rides along, once per wave and round (known before the products: it goes first)
        st_tagged(p.pss[kind] + ((((size_t)ring * kXcd + c.x) * kPer + c.j) * kCW + (threadIdx.x >> 6)) * 32 + (round & 1) * 16 + col,
                  ssrow[col], tag);
    // 64 bytes per (strip, row): lane (row, q) writes its four features 4q .. 4q + 3 as one 16-byte word, each
    // value with the word's parity in its lowest bit (see parity_bit); one store instruction per strip.  A
    // write-through store occupies the wave for ~0.3 us, several times the products of a strip: strip by
    // strip, so that a strip's store goes out while the next one is multiplied.
    const rsrc_t out = make_rsrc(p.part[kind]);
    const unsigned at8 = (unsigned)((((size_t)ring * kXcd + c.x) * p.nstrips[kind] + s0) * 16 + col) * 64u + kg * 16u;
#pragma unroll
    for (int si = 0; si < NSW; ++si) {
        f32x4 acc = (f32x4){0.f, 0.f, 0.f, 0.f}, acl = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kt = 0; kt < KTM; ++kt) {   // k-tiles beyond the XCD's slice: zero weights (their LDS columns are in bounds)
            const bf16x8 h = __builtin_bit_cast(bf16x8, *reinterpret_cast<const v4u*>(act_hi + at + kt * 32));
            const bf16x8 l = __builtin_bit_cast(bf16x8, *reinterpret_cast<const v4u*>(act_lo + at + kt * 32));
            const bf16x8 a = __builtin_bit_cast(bf16x8, w[si * KTM + kt]);
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, h, acc, 0, 0, 0);
            acl = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, l, acl, 0, 0, 0);
        }
        if (c.dbg && si == NSW - 1) {   // when tracing: the products are done (the stamp follows them in program order only through this)
            asm volatile("" :: "v"(acc), "v"(acl));
            stamp(c, dbg_stage, 3);
        }
        const f32x4 v = acc + acl;
        if (si < ns && col < p.MR)
            st_16(out, at8 + si * 1024u, (v4u){(__float_as_uint(v[0]) & ~1u) | pbit, (__float_as_uint(v[1]) & ~1u) | pbit,
                                               (__float_as_uint(v[2]) & ~1u) | pbit, (__float_as_uint(v[3]) & ~1u) | pbit});
    }
}

// Streamed kind: an IO wave tells the compute waves that its first requests for the stage input are out (see
// stream_stage) - behind them in program order, which is the order the unit serves requests in.
__device__ __forceinline__ void announce(unsigned* go) {
    __builtin_amdgcn_sched_barrier(0);
    if (go && (threadIdx.x & 63) == 0) atomicAdd(go, 1u);
    __builtin_amdgcn_sched_barrier(0);
}

// IO waves: copy the XCD's slice of a stage input (split planes [2][16][Kp], the first MR rows of each)
// from the XCD's buffer (byte offset `src` from the base of `r`) into LDS, which has the same layout:
// two contiguous runs of MR * Kp elements, up to NB 16-byte chunks per thread in flight.
template <int NB>
__device__ __forceinline__ void stage_copy(rsrc_t r, unsigned src, int MR, int Kp, uint16_t* act, int t, int nthreads,
                                           unsigned* go = nullptr) {
    const int per_plane = MR * Kp / 8, total = 2 * per_plane;   // Kp % 8 == 0
    const unsigned src_plane = 16u * (unsigned)Kp * 2u, dst_plane = (unsigned)MR * (unsigned)Kp * 2u;   // in LDS the planes hold MR rows only
    for (int base = 0; base < total; base += NB * nthreads) {
        v4u v[NB];
        unsigned at[NB];
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            const int q = base + i * nthreads + t;
            const bool second = q >= per_plane;
            const unsigned in_plane = (unsigned)(second ? q - per_plane : q) * 16u;
            at[i] = (second ? dst_plane : 0u) + in_plane;
            v[i] = q < total ? ld_16(r, src + (second ? src_plane : 0u) + in_plane) : (v4u){0u, 0u, 0u, 0u};
        }
        if (base == 0) announce(go);
#pragma unroll
        for (int i = 0; i < NB; ++i)
            if (base + i * nthreads + t < total) *reinterpret_cast<v4u*>(reinterpret_cast<char*>(act) + at[i]) = v[i];
    }
}

// The same for the 16-byte words [w0, w1) of every row only (the wide shape's W2 input goes to LDS in parts,
// one per chunk of 16 k-tiles, so that the products of the first part start while the rest is copied).
__device__ __forceinline__ void stage_copy_cols(rsrc_t r, unsigned src, int MR, int Kp, uint16_t* act, int t, int nthreads, int w0, int w1,
                                                unsigned* go) {
    const int wpr = w1 - w0, per_plane = MR * wpr, total = 2 * per_plane;
    const unsigned src_plane = 16u * (unsigned)Kp * 2u, dst_plane = (unsigned)MR * (unsigned)Kp * 2u;
    for (int base = 0; base < total; base += 8 * nthreads) {
        v4u v[8];
        unsigned at[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int q = base + i * nthreads + t;
            const bool second = q >= per_plane;
            const int qq = second ? q - per_plane : q, row = qq / wpr, w = qq - row * wpr;
            const unsigned in_plane = (unsigned)row * (unsigned)Kp * 2u + (unsigned)(w0 + w) * 16u;
            at[i] = (second ? dst_plane : 0u) + in_plane;
            v[i] = q < total ? ld_16(r, src + (second ? src_plane : 0u) + in_plane) : (v4u){0u, 0u, 0u, 0u};
        }
        if (base == 0) announce(go);
#pragma unroll
        for (int i = 0; i < 8; ++i)
            if (base + i * nthreads + t < total) *reinterpret_cast<v4u*>(reinterpret_cast<char*>(act) + at[i]) = v[i];
    }
}

// ------------------------------------------------------------------------- reduce jobs (IO waves)

// Sum of the eight XCDs' partials of strip s in accumulator layout (lane: rows 4 * (lane / 16) .. + 3
// of the strip = output features, column lane % 16 = activation row), added in XCD order.  scaled: the
// product follows a norm; the XCDs' shares of every row's sum of squares came with their partial sums,
// and *rn receives 1/rms of the lane's row.
// TWO: the partials of a second strip s2 (same product, -1: none) are polled along with the first's and
// their sum goes to *v2.
template <bool TWO = false>
__device__ __forceinline__ f32x4 gather_partials(const XP& p, Ctx& c, int kind, int s, int prod, int ring, unsigned tag, unsigned pbit,
                                                 int lane, bool scaled, float* rn, unsigned dbg_stage = 1000u, int s2 = -1,
                                                 f32x4* v2 = nullptr) {
    const int col = lane & 15, quad = lane >> 4;
    const bool live = col < p.MR;
    f32x4 val[kXcd];
#pragma unroll
    for (int x = 0; x < kXcd; ++x) val[x] = (f32x4){0.f, 0.f, 0.f, 0.f};
    unsigned need = live ? 0xFFu : 0u;
    f32x4 val2[TWO ? kXcd : 1];
    unsigned need2 = (TWO && live && s2 >= 0) ? 0xFFu : 0u;
    if (TWO) {
#pragma unroll
        for (int x = 0; x < kXcd; ++x) val2[x] = (f32x4){0.f, 0.f, 0.f, 0.f};
    }
    // (selects: indexing the kernel's parameter block with a run-time value is best avoided)
    const u64* part = kind == X_A ? p.part[X_A] : kind == X_C ? p.part[X_C] : kind == X_D ? p.part[X_D]
                                                                            : kind == X_E ? p.part[X_E] : p.part[X_LM];
    const u64* pssb = kind == X_A ? p.pss[X_A] : kind == X_D ? p.pss[X_D] : p.pss[X_LM];
    const int nstr = kind == X_A ? p.nstrips[X_A] : kind == X_C ? p.nstrips[X_C] : kind == X_D ? p.nstrips[X_D]
                                                                               : kind == X_E ? p.nstrips[X_E] : p.nstrips[X_LM];
    const rsrc_t in = make_rsrc(part);
    const unsigned at8 = (unsigned)(((size_t)ring * kXcd * nstr + s) * 16 + col) * 64u + quad * 16u;
    const unsigned xstride = (unsigned)nstr * 1024u;
    const unsigned at8b = at8 + (unsigned)((TWO ? s2 : s) - s) * 1024u;   // (the second strip's words)
    const unsigned pb = pbit * 0x1u;
    // sums of squares: the lane's quarter looks at XCDs 2 * quad and 2 * quad + 1; `prod` = the strip's
    // producer (unit * kCW + wave) * 2 + round, the same on every XCD
    const u64* pss = pssb + (((size_t)ring * kXcd + 2 * quad) * kPer * kCW * 2 + prod) * 16 + col;
    unsigned need_ss = (live && scaled) ? 3u : 0u;
    float ssv[2] = {0.f, 0.f};
    bool ok = c.dead;
    unsigned nspin = 0;
    for (unsigned spins = 0; spins < kSpinLimit && !ok; ++spins) {
        ++nspin;
        v4u w[kXcd], w2[TWO ? kXcd : 1];
        u64 sw[2] = {0ull, 0ull};
#pragma unroll
        for (int x = 0; x < kXcd; ++x)
            if ((need >> x) & 1u) w[x] = ld_16(in, at8 + x * xstride);
        if (TWO) {
#pragma unroll
            for (int x = 0; x < kXcd; ++x)
                if ((need2 >> x) & 1u) w2[x] = ld_16(in, at8b + x * xstride);
        }
#pragma unroll
        for (int i = 0; i < 2; ++i)
            if ((need_ss >> i) & 1u) sw[i] = ld_u64(pss + (size_t)i * kPer * kCW * 2 * 16);
#pragma unroll
        for (int x = 0; x < kXcd; ++x)
            if ((need >> x) & 1u) {
                if (((w[x][0] & w[x][1] & w[x][2] & w[x][3]) & 1u) == pb && ((w[x][0] | w[x][1] | w[x][2] | w[x][3]) & 1u) == pb) {
                    val[x] = (f32x4){__uint_as_float(w[x][0] & ~1u), __uint_as_float(w[x][1] & ~1u), __uint_as_float(w[x][2] & ~1u),
                                     __uint_as_float(w[x][3] & ~1u)};
                    need &= ~(1u << x);
                }
            }
#pragma unroll
        for (int i = 0; i < 2; ++i)
            if (((need_ss >> i) & 1u) && (unsigned)(sw[i] >> 32) == tag) {
                ssv[i] = __uint_as_float((unsigned)sw[i]);
                need_ss &= ~(1u << i);
            }
        if (TWO) {
#pragma unroll
            for (int x = 0; x < kXcd; ++x)
                if ((need2 >> x) & 1u) {
                    if (((w2[x][0] & w2[x][1] & w2[x][2] & w2[x][3]) & 1u) == pb && ((w2[x][0] | w2[x][1] | w2[x][2] | w2[x][3]) & 1u) == pb) {
                        val2[x] = (f32x4){__uint_as_float(w2[x][0] & ~1u), __uint_as_float(w2[x][1] & ~1u), __uint_as_float(w2[x][2] & ~1u),
                                          __uint_as_float(w2[x][3] & ~1u)};
                        need2 &= ~(1u << x);
                    }
                }
        }
        ok = __all(need == 0u && need_ss == 0u && need2 == 0u);
        if (!ok && (spins & 255u) == 255u && ld_u32(c.err) != 0u) break;
    }
    if (!ok) give_up(c);
    if (c.dbg && (threadIdx.x & 63) == 0 && (blockIdx.x == 0 || blockIdx.x == 248) && dbg_stage < 512u)
        c.dbg[((size_t)(blockIdx.x ? 1 : 0) * 512 + dbg_stage) * 16 + 14] = nspin;
    if (scaled) {
        float a = ssv[0] + ssv[1];
        a = sum_xor16(a);
        a = sum_xor32(a);
        *rn = 1.0f / sqrtf(a / (float)p.d + p.eps);
    }
    f32x4 v = val[0];
#pragma unroll
    for (int x = 1; x < kXcd; ++x) v += val[x];
    if (TWO) {
        f32x4 u = val2[0];
#pragma unroll
        for (int x = 1; x < kXcd; ++x) u += val2[x];
        *v2 = u;
    }
    return v;
}

// Publishes a strip of the residual stream for the product that follows a norm: the values times the
// norm's gain as split planes, and the strip's sums of squares, into the owner XCD's buffer (ring slot
// `ring`; which = 0: x -> region o_a, 1: x' -> region o_x2).
__device__ __forceinline__ void put_stream(const XP& p, const Ctx& c, int which, int ring, int strip, int lane, f32x4 x, uint2 gain) {
    const int col = lane & 15, quad = lane >> 4;
    const bool live = col < p.MR;
    float s2 = live ? x[0] * x[0] + x[1] * x[1] + x[2] * x[2] + x[3] * x[3] : 0.f;
    s2 = sum_xor16(s2);
    s2 = sum_xor32(s2);
    uint8_t* buf = xcd_buf(p, c.x, ring);
    if (live) {
        const int per_xcd = p.d / 16 / kXcd;
        uint16_t* hi = reinterpret_cast<uint16_t*>(buf + (which ? p.o_x2 : p.o_a));
        uint16_t* lo = hi + (size_t)16 * p.KpA;
        const size_t at = (size_t)col * p.KpA + (strip % per_xcd) * 16 + 4 * quad;
        put_split4(hi + at, lo + at, times_gain(x, gain));
        if (quad == 0) reinterpret_cast<float*>(buf + p.o_ss)[((size_t)which * per_xcd + strip % per_xcd) * 16 + col] = s2;
    }
}
// What an IO wave does in every layer, read from the tables once at kernel start: its reduce job of
// each kind (strip, flag slot; strip < 0: none), the lane's row of the step, the rotary factors of
// its QKV strip, the number of flag words each stage's consumers wait for, the unit's attention job.
struct IoJobs {
    int sD2;                     // second W1|W3 strip of the wave (shapes with more such strips than IO waves; -1: none)
    int sA, sC, sD, sE;          // strip of the wave's reduce job of each product (named fields, not arrays: a select
    int tA, tC, tD, tE;          // between array elements by a run-time value would be turned into memory indexing); flag slots
    RowPos rp;                   // row lane % 16 of the step
    float2 rot0, rot1;           // QKV strip: cos, sin of the lane's two rotary pairs at the row's position
    int nA, nB, nC, nD, nE;      // flag words the consumers of stage A (reduce of QKV), B (attention), C, D, E wait for
    int a_seq, a_h, a_rg, a_slot;   // attention job of the unit (a_rg < 0: none)
    int pA, pD;                  // producers (see gather_partials) of the wave's QKV and W1|W3 strips
    int a_ke, a_kv0;             // ... its sequence's draft length this step and the positions cached before this launch
                                 // (read here once: fetched at every attention stage they would add a memory round trip
                                 // to every layer's critical path)
};
template <int HD>
__device__ __forceinline__ IoJobs load_io_jobs(const XP& p, const Ctx& c, int io, int lane) {
    IoJobs j;
    auto entry = [&](int k) { return p.rtab + ((((size_t)k * kXcd + c.x) * kPer + c.j) * kNIO + io) * 3; };
    j.sA = entry(X_A)[0]; j.tA = entry(X_A)[1];
    j.sC = entry(X_C)[0]; j.tC = entry(X_C)[1];
    j.sD = entry(X_D)[0]; j.tD = entry(X_D)[1]; j.sD2 = HD == 64 ? -1 : entry(X_D)[2];   // (second strips: the wide shape only)
    j.sE = entry(X_E)[0]; j.tE = entry(X_E)[1];
    const int col = lane & 15, quad = lane >> 4;
    j.rp = col < p.MR ? row_pos(p, col) : RowPos{0, 0, 0, 0, false};
    j.rot0 = j.rot1 = make_float2(1.f, 0.f);
    if (j.sA >= 0 && col < p.MR) {
        const int o0 = j.sA * 16, seg = o0 / p.d, j0 = o0 - seg * p.d;
        if (seg < 2) {
            const float2* rt = p.rope + (size_t)j.rp.pos * (HD / 2) + ((j0 % HD) >> 1) + 2 * quad;
            j.rot0 = rt[0];
            j.rot1 = rt[1];
        }
    }
    j.nA = p.njobs[F_A][c.x]; j.nB = p.njobs[F_B][c.x]; j.nC = p.njobs[F_C][c.x]; j.nD = p.njobs[F_D][c.x];
    j.nE = p.njobs[F_E][c.x];
    const int16_t* a = p.atab + ((size_t)c.x * kPer + c.j) * 4;
    j.a_seq = a[0]; j.a_h = a[1]; j.a_rg = a[2]; j.a_slot = a[3];
    j.pA = j.sA >= 0 ? p.ptab[p.poff[X_A] + j.sA] : 0;
    j.pD = j.sD >= 0 ? p.ptab[p.poff[X_D] + j.sD] : 0;
    j.a_ke = -1; j.a_kv0 = 0;
    if (j.a_rg >= 0) {
        const int b = j.a_seq % p.B;
        j.a_ke = p.k_eff[b];
        j.a_kv0 = j.a_ke >= 0 ? p.C + p.n[b] - 1 : 0;
    }
    return j;
}

// The reduce job of an IO wave for product `kind` (X_A .. X_E, a run-time value: the four products share
// one copy of this code, which keeps the kernel inside the instruction cache) of `layer`; none: returns
// at once.  resid: the wave's strip of the residual stream (owners of Wo / W2 strips).
template <int HD>
__device__ __forceinline__ void reduce_job(const XP& p, Ctx& c, const IoJobs& jb, int kind, int layer, int lane, f32x4& resid,
                                           unsigned stage) {
    // (selects, not indexing with a run-time value: that would move the structure into memory)
    const int s = kind == X_A ? jb.sA : kind == X_C ? jb.sC : kind == X_D ? jb.sD : jb.sE;
    const int slot = kind == X_A ? jb.tA : kind == X_C ? jb.tC : kind == X_D ? jb.tD : jb.tE;
    // the wide shape has more W1|W3 strips than IO waves: a wave's second strip is gathered along with its first
    const int s2 = (HD != 64 && kind == X_D) ? jb.sD2 : -1;
    if (s < 0) return;
    const int col = lane & 15, quad = lane >> 4, d = p.d, ring = layer & 1;
    const bool live = col < p.MR;
    const int flag = kind == X_A ? F_A : kind == X_C ? F_C : kind == X_D ? F_D : F_E;
    const unsigned tag = tag_of(c, layer, flag);
    uint8_t* buf = xcd_buf(p, c.x, ring);
    const bool scaled = kind == X_A || kind == X_D;   // QKV and W1|W3 follow a norm
    uint2 gain = make_uint2(0u, 0u);   // Wo, W2: gain of the norm that follows, for the lane's four features
    if (kind == X_C) gain = *reinterpret_cast<const uint2*>(p.blob + (p.g2_off + (u64)layer * p.layer_bytes) / 2 + s * 16 + 4 * quad);
    if (kind == X_E) {
        const uint16_t* g = layer + 1 < p.L ? p.blob + (p.g1_off + (u64)(layer + 1) * p.layer_bytes) / 2 : p.blob + p.gf_off / 2;
        gain = *reinterpret_cast<const uint2*>(g + s * 16 + 4 * quad);
    }
    float rn = 1.f;
    f32x4 v, vb = (f32x4){0.f, 0.f, 0.f, 0.f};
    if (HD != 64 && kind == X_D)
        v = gather_partials<true>(p, c, kind, s, jb.pD, ring, tag, parity_bit(c, kind, layer, col), lane, scaled, &rn,
                                  stage, s2, &vb);
    else
        v = gather_partials(p, c, kind, s, kind == X_A ? jb.pA : kind == X_D ? jb.pD : 0, ring, tag, parity_bit(c, kind, layer, col), lane,
                            scaled, &rn, stage);
    stamp(c, stage, 4);
    v *= rn;
    stamp(c, stage, 5);
    if (kind == X_A) {
        const int seg = (s * 16) / d, j0 = s * 16 - seg * d, h = j0 / HD;
        const float a0 = v[0] * jb.rot0.x - v[1] * jb.rot0.y, b0 = v[0] * jb.rot0.y + v[1] * jb.rot0.x;
        const float a1 = v[2] * jb.rot1.x - v[3] * jb.rot1.y, b1 = v[2] * jb.rot1.y + v[3] * jb.rot1.x;
        if (live) {
            const int hl = h - p.hd0[c.x], f0 = j0 % HD + 4 * quad;   // head among the XCD's, first of the lane's four features
            if (seg == 0) {   // queries of this XCD's heads, scaled by 1 / sqrt(head dimension): {value, tag} pairs
                v4u* q = reinterpret_cast<v4u*>(buf + p.o_q + ((size_t)col * (p.KpO - 8) + hl * HD + f0) * 8);
                q[0] = (v4u){__float_as_uint(a0 * (HD == 64 ? 0.125f : 0.08838834764831845f)), tag, __float_as_uint(b0 * (HD == 64 ? 0.125f : 0.08838834764831845f)), tag};
                q[1] = (v4u){__float_as_uint(a1 * (HD == 64 ? 0.125f : 0.08838834764831845f)), tag, __float_as_uint(b1 * (HD == 64 ? 0.125f : 0.08838834764831845f)), tag};
            } else {
                // keys (rotated) / values as fp16 pairs: into the cache for the steps to come (valid rows), and
                // as tagged pairs for this launch's attention jobs, which poll them ({pair, tag, pair, tag})
                const _Float16 h0 = (_Float16)a0, h1 = (_Float16)b0, h2 = (_Float16)a1, h3 = (_Float16)b1;
                const unsigned p01 = (unsigned)__builtin_bit_cast(unsigned short, h0) | ((unsigned)__builtin_bit_cast(unsigned short, h1) << 16);
                const unsigned p23 = (unsigned)__builtin_bit_cast(unsigned short, h2) | ((unsigned)__builtin_bit_cast(unsigned short, h3) << 16);
                if (jb.rp.valid) {
                    _Float16* dst = (seg == 1 ? p.Kc : p.Vc) +
                                    ((((size_t)layer * p.Smax + jb.rp.seq) * p.H + h) * p.Tmax + jb.rp.slot) * HD + f0;
                    *reinterpret_cast<uint2*>(dst) = make_uint2(p01, p23);
                }
                *reinterpret_cast<v4u*>(buf + p.o_kv + ((((size_t)(seg - 1) * 16 + col) * ((p.KpO - 8) / HD) + hl) * (HD / 4) + f0 / 4) * 16) =
                    (v4u){p01, tag, p23, tag};
            }
        }
    } else if (kind == X_D) {   // rows 0..7 of the strip: W1 rows s * 8 + i, rows 8..15 the matching W3 rows
        auto swiglu = [&](f32x4 w, int strip) {
            f32x4 u3;
#pragma unroll
            for (int e = 0; e < 4; ++e) u3[e] = lane_xor32(w[e]);
            if (live && quad < 2) {
                f32x4 hv;
#pragma unroll
                for (int e = 0; e < 4; ++e) hv[e] = w[e] / (1.0f + expf(-w[e])) * u3[e];
                uint16_t* hi = reinterpret_cast<uint16_t*>(buf + p.o_h);
                uint16_t* lo = hi + (size_t)16 * p.KpH;
                const size_t at = (size_t)col * p.KpH + (strip * 8 - p.ke0[c.x] * 32) + 4 * quad;
                put_split4(hi + at, lo + at, hv);
            }
        };
        swiglu(v, s);
        if (HD != 64 && s2 >= 0) swiglu(vb * rn, s2);
    } else {   // Wo: x' = x + Wo o; W2: x (next layer) = x' + W2 h - published times the gain of the norm that follows
        resid += v;
        const int out_ring = kind == X_C ? ring : (layer + 1) & 1;
        put_stream(p, c, kind == X_C, out_ring, s, lane, resid, gain);
        if (kind == X_E && layer == p.L - 1 && live)   // final hidden rows, for the kernels that follow
            *reinterpret_cast<f32x4*>(p.X + (size_t)col * d + s * 16 + 4 * quad) = resid;
    }
    if (kind != X_A) raise_flag(p, c, flag, slot, tag);   // (queries, keys and values carry their own tags)
}

// Output projection: logits of the strip's 16 vocabulary entries for every row.
__device__ __forceinline__ void reduce_logits(const XP& p, Ctx& c, int io, int lane) {
    const int col = lane & 15, quad = lane >> 4;
    const unsigned tag = tag_of(c, p.L, F_A);
    for (int i = 0;; ++i) {   // strips (i * 32 * kNIO + unit * kNIO + io) * 8 + XCD of the output projection
        const int s = ((i * kPer + (int)c.j) * kNIO + io) * kXcd + (int)c.x;
        if (s >= p.nstrips[X_LM]) break;
        float rn = 1.f;
        const f32x4 v = gather_partials(p, c, X_LM, s, p.ptab[p.poff[X_LM] + s], 0, tag, parity_bit(c, X_LM, 0, col), lane, true, &rn) * rn;
        if (col < p.MR) *reinterpret_cast<f32x4*>(p.logit_s + (size_t)col * p.Vs + s * 16 + 4 * quad) = v;
    }
}

// ------------------------------------------------------------------------- attention (as one unit's job)

// A lane's share of one row's attention: the weighted sum over its 8 * NCH features, running maximum, denominator.
template <int NCH>
struct AttnAcc { float acc[8 * NCH], mx, den; };

__device__ __forceinline__ float sum8(float v) {
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xB1, 0xF, 0xF, true));
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x4E, 0xF, 0xF, true));
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x141, 0xF, 0xF, true));
    return v;
}
__device__ __forceinline__ void halves8(v4u raw, float* f) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        f[2 * e] = (float)__builtin_bit_cast(_Float16, (unsigned short)(raw[e] & 0xFFFFu));
        f[2 * e + 1] = (float)__builtin_bit_cast(_Float16, (unsigned short)(raw[e] >> 16));
    }
}

// Eight lanes share a cache position; lane dg of them holds features 64 c + 8 dg .. + 7 of every 64-feature
// chunk c of the head (NCH chunks: one 16-byte load each).
//
// One cache position per lane group; row r0 + r of the sequence sees it iff bit r0 + r of vis is set.
template <int RPJ, int NCH>
__device__ __forceinline__ void attend(const float (&q)[RPJ][8 * NCH], int r0, const v4u (&kraw)[NCH], const v4u (&vraw)[NCH], unsigned vis,
                                       int ke, AttnAcc<NCH> (&A)[RPJ]) {
    float kf[8 * NCH], vf[8 * NCH];
#pragma unroll
    for (int ch = 0; ch < NCH; ++ch) {
        halves8(kraw[ch], kf + 8 * ch);
        halves8(vraw[ch], vf + 8 * ch);
    }
#pragma unroll
    for (int r = 0; r < RPJ; ++r) {
        float sc = 0.f;
#pragma unroll
        for (int e = 0; e < 8 * NCH; ++e) sc += q[r][e] * kf[e];
        sc = sum8(sc);
        if (((vis >> (r0 + r)) & 1u) && r0 + r <= ke) {
            const float mn = fmaxf(A[r].mx, sc);
            const float corr = __expf(A[r].mx - mn), pw = __expf(sc - mn);
            A[r].den = A[r].den * corr + pw;
#pragma unroll
            for (int e = 0; e < 8 * NCH; ++e) A[r].acc[e] = A[r].acc[e] * corr + pw * vf[e];
            A[r].mx = mn;
        }
    }
}

// NIT cache positions per lane group at once: all scores, one running-maximum update per row, then
// the weighted values.
template <int RPJ, int NCH, int NIT>
__device__ __forceinline__ void attend_round(const float (&q)[RPJ][8 * NCH], int r0, const v4u (&kk)[NIT * NCH], const v4u (&vv)[NIT * NCH],
                                             int pos0, int stride, int o1, int ke, AttnAcc<NCH> (&A)[RPJ]) {
    float sc[RPJ][NIT];
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
        float kf[8 * NCH];
#pragma unroll
        for (int ch = 0; ch < NCH; ++ch) halves8(kk[it * NCH + ch], kf + 8 * ch);
        const bool on = pos0 + it * stride < o1;
#pragma unroll
        for (int r = 0; r < RPJ; ++r) {
            float dd = 0.f;
#pragma unroll
            for (int e = 0; e < 8 * NCH; ++e) dd += q[r][e] * kf[e];
            dd = sum8(dd);
            sc[r][it] = (on && r0 + r <= ke) ? dd : -1e30f;
        }
    }
#pragma unroll
    for (int r = 0; r < RPJ; ++r) {
        float mn = A[r].mx;
#pragma unroll
        for (int it = 0; it < NIT; ++it) mn = fmaxf(mn, sc[r][it]);
        const float corr = __expf(A[r].mx - mn);
        float sum = 0.f;
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            sc[r][it] = sc[r][it] > -1e29f ? __expf(sc[r][it] - mn) : 0.f;
            sum += sc[r][it];
        }
        A[r].den = A[r].den * corr + sum;
        A[r].mx = mn;
#pragma unroll
        for (int e = 0; e < 8 * NCH; ++e) A[r].acc[e] *= corr;
    }
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
        float vf[8 * NCH];
#pragma unroll
        for (int ch = 0; ch < NCH; ++ch) halves8(vv[it * NCH + ch], vf + 8 * ch);
#pragma unroll
        for (int r = 0; r < RPJ; ++r)
#pragma unroll
            for (int e = 0; e < 8 * NCH; ++e) A[r].acc[e] += sc[r][it] * vf[e];
    }
}

struct Lds {
    unsigned* join;     // arrivals of the IO waves at their own barrier (only ever grows)
    unsigned* go;       // streamed kind: IO waves that have requested a stage input, counted over the launch (a hint, see stream_stage)
    uint16_t* act0;     // staged K-slices, alternating between stages: hi plane, lo plane behind it; odd stages use
    unsigned act_elems; //   the buffer act_elems elements further on (an offset, not a second pointer to choose from: a
                        //   select between members by a run-time value tends to end up as indexing in memory)
    float* ss0;         // sums of squares of the XCD's slice of the stage input, per row; odd stages 16 floats further on
    float* part;        // attention: [kNIO][RPJ][hd + 4] partial rows of the IO waves (outputs, max, sum, pad)
    float* qs;          // attention: [RPJ][hd] scaled queries
};

// Attention of one (sequence, head, row group) on the XCD that owns the head: the cached positions
// (requested before the queries are there) and the rows appended by this launch.  The unit's compute
// waves run attn_compute, its IO waves attn_io; both cross the same two workgroup barriers.

// Workgroup barrier that orders LDS traffic only: the waves' own LDS accesses are done, nothing is said
// about global memory (a full barrier would also wait for every weight tile in flight, including those
// requested for later stages).
__device__ __forceinline__ void lds_barrier() {
    compiler_fence();
    __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0)
    __builtin_amdgcn_s_barrier();
    compiler_fence();
}

// Barrier of the unit's IO waves alone (LDS counter; the compute waves are busy fetching weights).
// `joins`: barriers of this kind the wave has crossed so far.
__device__ __forceinline__ void io_barrier(const Lds& s, unsigned& joins, int lane) {
    const unsigned want = ++joins * kNIO;
    __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0): the wave's LDS writes are done
    if (lane == 0) atomicAdd(s.join, 1u);
    for (unsigned spins = 0; spins < kSpinLimit; ++spins) {
        if ((int)(__hip_atomic_load(s.join, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) - want) >= 0) break;
        __builtin_amdgcn_s_sleep(1);
    }
    compiler_fence();
}

// Runs on the unit's four IO waves (they hold no weights): each takes a quarter of the cached positions.
template <int RPJ, int HD = 64>
__device__ __forceinline__ void attn_io(const XP& p, Ctx& c, const IoJobs& jb, const Lds& s, int layer, unsigned stage,
                                        unsigned& joins) {
    if (jb.a_rg < 0) return;   // this unit has no job (the same for all its waves)
    const int io = (threadIdx.x >> 6) - kCW, lane = threadIdx.x & 63;
    const int seq = jb.a_seq, h = jb.a_h, RS = p.RS, r0 = jb.a_rg * RPJ;
    // lanes per cache position, positions per wave and look, 64-feature chunks of a head, positions per lane group
    // and register buffer, floats per partial row
    constexpr int LPP = 8, PPW = 64 / LPP, NCH = HD / 64, NIT = kNIT / NCH, PS = HD + 4;
    const int pg = lane / LPP, dg = lane % LPP;
    const int ke = jb.a_ke, kv0 = jb.a_kv0;   // draft length of the sequence's prompt; positions cached before this launch
    const int nrounds = (kv0 + NIT * kNIO * PPW - 1) / (NIT * kNIO * PPW);
    const size_t head0 = ((((size_t)layer * p.Smax + seq) * p.H + h) * p.Tmax) * HD;   // the head's entries, contiguous
    // The head's cached keys / values through buffer resources that end at the cached length: requests past it
    // (the tail of the last round, rounds asked for beyond the last) are answered with zeros and move nothing,
    // so the requests need no branches - with loads under branches every wait would be for all of them.
    auto head_rsrc = [&](const _Float16* base) {
        const u64 a = reinterpret_cast<u64>(base + head0);   // the job is the unit's: the same in every lane
        const u64 u = uniform64(a);
        return __builtin_amdgcn_make_buffer_rsrc(reinterpret_cast<void*>(u), 0, __builtin_amdgcn_readfirstlane(kv0 * HD * 2), 0x00020000);
    };
    const rsrc_t Kr = head_rsrc(p.Kc), Vr = head_rsrc(p.Vc);
    const unsigned tag = tag_of(c, layer, F_B);
    uint8_t* buf = xcd_buf(p, c.x, layer & 1);
    v4u ka[kNIT], va[kNIT], kb[kNIT], vb[kNIT], kc[kNIT], vc[kNIT];   // three rounds in flight (kNIT = NIT * NCH loads each)
    auto fetch = [&](v4u (&kk)[kNIT], v4u (&vv)[kNIT], int rnd) {
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            const unsigned at = (unsigned)(((rnd * NIT + it) * (kNIO * PPW) + io * PPW + pg) * HD + dg * 8) * 2u;
#pragma unroll
            for (int ch = 0; ch < NCH; ++ch) {
                vv[it * NCH + ch] = __builtin_amdgcn_raw_buffer_load_b128(Vr, at + ch * 128u, 0, 0);
                kk[it * NCH + ch] = __builtin_amdgcn_raw_buffer_load_b128(Kr, at + ch * 128u, 0, 0);
            }
        }
    };
    stamp(c, stage, 0);
    fetch(ka, va, 0);
    fetch(kb, vb, 1);
    fetch(kc, vc, 2);
    const unsigned tagA = tag_of(c, layer, F_A);   // what the reduce jobs of the QKV product wrote carries this tag
    if (io == 0) {   // the job's queries: polled where the reduce jobs put them
        constexpr int QL = HD / 64;   // query values per lane
        const u64* q = reinterpret_cast<const u64*>(buf + p.o_q) + (size_t)(seq * RS + r0) * (p.KpO - 8) + (h - p.hd0[c.x]) * HD + lane;
        u64 qv[RPJ][QL];
        unsigned pend = 0u;
#pragma unroll
        for (int r = 0; r < RPJ; ++r) {
#pragma unroll
            for (int e = 0; e < QL; ++e) {
                qv[r][e] = 0ull;
                if (r0 + r < RS && !c.dead) pend |= 1u << (r * QL + e);
            }
        }
        bool ok = false;
        for (unsigned spins = 0; spins < kSpinLimit && !ok; ++spins) {
#pragma unroll
            for (int r = 0; r < RPJ; ++r)
#pragma unroll
                for (int e = 0; e < QL; ++e)
                    if ((pend >> (r * QL + e)) & 1u) qv[r][e] = ld_u64(q + (size_t)r * (p.KpO - 8) + 64 * e);
#pragma unroll
            for (int r = 0; r < RPJ; ++r)
#pragma unroll
                for (int e = 0; e < QL; ++e)
                    if (((pend >> (r * QL + e)) & 1u) && (unsigned)(qv[r][e] >> 32) == tagA) pend &= ~(1u << (r * QL + e));
            ok = __all(pend == 0u);
            if (!ok && (spins & 255u) == 255u && ld_u32(c.err) != 0u) break;
        }
        if (!ok) give_up(c);
        stamp(c, stage, 1);
#pragma unroll
        for (int r = 0; r < RPJ; ++r)
#pragma unroll
            for (int e = 0; e < QL; ++e)
                s.qs[r * HD + lane + 64 * e] = (r0 + r < RS && ok) ? __uint_as_float((unsigned)qv[r][e]) : 0.f;
    }
    io_barrier(s, joins, lane);   // the queries are in LDS
    if (io == 0) stamp(c, stage, 3);
    {
        AttnAcc<NCH> A[RPJ];
#pragma unroll
        for (int r = 0; r < RPJ; ++r) {
            A[r].mx = -1e30f; A[r].den = 0.f;
#pragma unroll
            for (int e = 0; e < 8 * NCH; ++e) A[r].acc[e] = 0.f;
        }
        float q[RPJ][8 * NCH];
#pragma unroll
        for (int r = 0; r < RPJ; ++r) {
#pragma unroll
            for (int ch = 0; ch < NCH; ++ch) {
                const float4 qa = *reinterpret_cast<const float4*>(s.qs + r * HD + ch * 64 + dg * 8);
                const float4 qb = *reinterpret_cast<const float4*>(s.qs + r * HD + ch * 64 + dg * 8 + 4);
                q[r][8 * ch + 0] = qa.x; q[r][8 * ch + 1] = qa.y; q[r][8 * ch + 2] = qa.z; q[r][8 * ch + 3] = qa.w;
                q[r][8 * ch + 4] = qb.x; q[r][8 * ch + 5] = qb.y; q[r][8 * ch + 6] = qb.z; q[r][8 * ch + 7] = qb.w;
            }
        }
        auto run = [&](const v4u (&kk)[kNIT], const v4u (&vv)[kNIT], int rnd) {
            const int pos0 = rnd * NIT * (kNIO * PPW) + io * PPW + pg;
            attend_round<RPJ, NCH, NIT>(q, r0, kk, vv, pos0, kNIO * PPW, kv0, ke, A);
        };
        // Rows appended by this launch (up to 16: lane group pg takes rows pg and pg + 8), polled as the tagged
        // fp16 pairs this XCD's reduce jobs write.  Who sees them: in a chain row r sees row a iff a <= r, in a
        // candidate tree iff a is r itself or an ancestor.  Row pg is requested now and used after the cached
        // positions; row pg + 8 (trees of more than 8 nodes only) is fetched behind them.
        auto seen_by = [&](int a) {
            unsigned vis = 0u;
            if (io == 0 && a <= ke && a < RS) {
#pragma unroll
                for (int r = 0; r < RPJ; ++r) {
                    const int row = r0 + r;
                    const bool sees = p.tanc ? (row == a || ((p.tanc[min(row, 15)] >> a) & 1ull)) : a <= row;
                    if (row < RS && sees) vis |= 1u << row;
                }
            }
            return vis;
        };
        auto fetch_row = [&](int a, unsigned& vis, v4u (&kn)[NCH], v4u (&vn)[NCH]) {   // lane dg = features 64 ch + 8 dg .. + 7
            const rsrc_t kvr = make_rsrc(p.xbuf);
            const unsigned hw = (unsigned)(p.KpO - 8) / (unsigned)HD;   // heads a row of the region has room for
            const unsigned atk = (unsigned)(((size_t)c.x * kRing + (layer & 1)) * p.xcd_bytes + p.o_kv) +
                                 ((((unsigned)(seq * RS + a)) * hw + (unsigned)(h - p.hd0[c.x])) * (unsigned)(HD / 4) + 2u * dg) * 16u;
            const unsigned atv = atk + 16u * hw * (unsigned)(HD / 4) * 16u;
            v4u k0[NCH], k1[NCH], v0[NCH], v1[NCH];
            bool ok = vis == 0u || c.dead;   // rows nobody of this job sees are not waited for
            for (unsigned spins = 0; spins < kSpinLimit && !__all(ok); ++spins) {
                if (!ok) {
                    ok = true;
#pragma unroll
                    for (int ch = 0; ch < NCH; ++ch) {   // (a chunk's 64 features: 16 words of 16 bytes)
                        k0[ch] = ld_16(kvr, atk + ch * 256u); k1[ch] = ld_16(kvr, atk + ch * 256u + 16u);
                        v0[ch] = ld_16(kvr, atv + ch * 256u); v1[ch] = ld_16(kvr, atv + ch * 256u + 16u);
                    }
#pragma unroll
                    for (int ch = 0; ch < NCH; ++ch)
                        ok = ok && k0[ch][1] == tagA && k0[ch][3] == tagA && k1[ch][1] == tagA && k1[ch][3] == tagA &&
                             v0[ch][1] == tagA && v0[ch][3] == tagA && v1[ch][1] == tagA && v1[ch][3] == tagA;
                    if (ok) {
#pragma unroll
                        for (int ch = 0; ch < NCH; ++ch) {
                            kn[ch] = (v4u){k0[ch][0], k0[ch][2], k1[ch][0], k1[ch][2]};
                            vn[ch] = (v4u){v0[ch][0], v0[ch][2], v1[ch][0], v1[ch][2]};
                        }
                    }
                }
                if ((spins & 255u) == 255u && ld_u32(c.err) != 0u) break;
            }
            if (!__all(ok)) { give_up(c); vis = 0u; }
        };
        v4u kn[NCH], vn[NCH];
#pragma unroll
        for (int ch = 0; ch < NCH; ++ch) kn[ch] = vn[ch] = (v4u){0u, 0u, 0u, 0u};
        unsigned vis0 = seen_by(pg);
        if (io == 0) fetch_row(pg, vis0, kn, vn);
        // (nothing pending on entry: otherwise the wait at the loop's head is taken for both ways into it, as a wait
        // for every request - those of the two rounds that should stay in flight included)
        __builtin_amdgcn_s_waitcnt(0x0f70);   // vmcnt(0)
        // Requests are made for rounds past the last as well: zeros, nothing moves.  The fences keep a refill
        // behind the last use of the registers it fills: moved ahead of it, it would go to other registers and be
        // copied at the loop's end, behind a wait for every request.
        if constexpr (HD == 64) {
            // Whole trips of three rounds in the loop, straight-line code (with branches in it, the waits inside
            // fall back to waits for every request); the last one or two rounds behind it.
            int rnd = 0;
            for (; rnd + 3 <= nrounds; rnd += 3) {
                run(ka, va, rnd);
                __builtin_amdgcn_sched_barrier(0);
                fetch(ka, va, rnd + 3);
                __builtin_amdgcn_sched_barrier(0);
                run(kb, vb, rnd + 1);
                __builtin_amdgcn_sched_barrier(0);
                fetch(kb, vb, rnd + 4);
                __builtin_amdgcn_sched_barrier(0);
                run(kc, vc, rnd + 2);
                __builtin_amdgcn_sched_barrier(0);
                fetch(kc, vc, rnd + 5);
            }
            if (rnd < nrounds) run(ka, va, rnd);
            if (rnd + 1 < nrounds) run(kb, vb, rnd + 1);
        } else {
            // The wide heads: a round's products are long and the registers full - the rounds past the last are
            // skipped inside the loop (the two extra copies of the products that a tail needs cost 40 spilled
            // registers here, and 4 % of the kernel).
            for (int rnd = 0; rnd < nrounds; rnd += 3) {
                run(ka, va, rnd);
                __builtin_amdgcn_sched_barrier(0);
                fetch(ka, va, rnd + 3);
                __builtin_amdgcn_sched_barrier(0);
                if (rnd + 1 < nrounds) run(kb, vb, rnd + 1);
                __builtin_amdgcn_sched_barrier(0);
                fetch(kb, vb, rnd + 4);
                __builtin_amdgcn_sched_barrier(0);
                if (rnd + 2 < nrounds) run(kc, vc, rnd + 2);
                __builtin_amdgcn_sched_barrier(0);
                fetch(kc, vc, rnd + 5);
            }
        }
        if (io == 0) stamp(c, stage, 4);
        if (vis0) attend<RPJ, NCH>(q, r0, kn, vn, vis0, ke, A);
        for (int a = pg + PPW; a - pg < RS; a += PPW) {   // (the trip count is uniform over the launch)
            unsigned vis1 = seen_by(a);
            if (io == 0) fetch_row(a, vis1, kn, vn);
            if (vis1) attend<RPJ, NCH>(q, r0, kn, vn, vis1, ke, A);
        }
        if (io == 0) stamp(c, stage, 5);
#pragma unroll
        for (int r = 0; r < RPJ; ++r) {
#pragma unroll
            for (int o = LPP; o < 64; o <<= 1) {
                auto other = [&](float xx) { return o == 8 ? lane_xor8(xx) : (o == 16 ? lane_xor16(xx) : lane_xor32(xx)); };
                const float omx = other(A[r].mx), oden = other(A[r].den);
                const float mn = fmaxf(A[r].mx, omx);
                const float f0 = __expf(A[r].mx - mn), f1 = __expf(omx - mn);
                A[r].den = A[r].den * f0 + oden * f1;
#pragma unroll
                for (int e = 0; e < 8 * NCH; ++e) A[r].acc[e] = A[r].acc[e] * f0 + other(A[r].acc[e]) * f1;
                A[r].mx = mn;
            }
            if (pg == 0) {
                float* mine = s.part + ((size_t)io * RPJ + r) * PS;
#pragma unroll
                for (int ch = 0; ch < NCH; ++ch) {
                    const float* a8 = A[r].acc + 8 * ch;
                    *reinterpret_cast<float4*>(mine + ch * 64 + dg * 8) = make_float4(a8[0], a8[1], a8[2], a8[3]);
                    *reinterpret_cast<float4*>(mine + ch * 64 + dg * 8 + 4) = make_float4(a8[4], a8[5], a8[6], a8[7]);
                }
                if (dg == 0) *reinterpret_cast<float2*>(mine + HD) = make_float2(A[r].mx, A[r].den);
            }
        }
    }
    io_barrier(s, joins, lane);   // the waves' partial rows are in LDS
    if (io == 0) stamp(c, stage, 6);
    if (io == 0) {   // merge them; lane: row lane / 16 of the job, dims 4 * (lane % 16) .. + 3
        const int r = lane / (HD / 4), q4 = lane % (HD / 4);
        if (r < RPJ && r0 + r < RS) {
            float m2 = -1e30f;
#pragma unroll
            for (int w = 0; w < kNIO; ++w) m2 = fmaxf(m2, s.part[((size_t)w * RPJ + r) * PS + HD]);
            float dn = 0.f;
            f32x4 o = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int w = 0; w < kNIO; ++w) {
                const float* src = s.part + ((size_t)w * RPJ + r) * PS;
                const float f = __expf(src[HD] - m2);
                dn += src[HD + 1] * f;
                o += *reinterpret_cast<const f32x4*>(src + 4 * q4) * f;
            }
            const float inv = dn > 0.f ? 1.0f / dn : 0.f;
            uint16_t* hi = reinterpret_cast<uint16_t*>(buf + p.o_o);
            uint16_t* lo = hi + (size_t)16 * p.KpO;
            const size_t at = (size_t)(seq * RS + r0 + r) * p.KpO + (h - p.hd0[c.x]) * HD + 4 * q4;
            put_split4(hi + at, lo + at, o * inv);
        }
        raise_flag(p, c, F_B, jb.a_slot, tag);
        stamp(c, stage, 2);
    }
}

// ------------------------------------------------------------------------- one matrix-product stage

__device__ __forceinline__ unsigned product_tag(const XP& p, const Ctx& c, int kind, int layer) {
    return kind == X_LM ? tag_of(c, p.L, F_A)
                        : tag_of(c, layer, kind == X_A ? F_A : kind == X_C ? F_C : kind == X_D ? F_D : F_E);
}

// Compute waves.  KIND: which matrix; NSW: strips per wave and round; KTM: most k-tiles an XCD's slice
// has.  w holds this stage's tiles, requested one or two stages ago.
template <int KIND, int NSW, int KTM, class Prefetch>
__device__ __forceinline__ void compute_stage(const XP& p, const Ctx& c, const GJob& g, const Lds& s, int layer, unsigned stage,
                                              int Kp, v4u (&w)[NSW * KTM], Prefetch&& prefetch) {
    const int lane = threadIdx.x & 63;
    const uint16_t* act_hi = s.act0 + (size_t)(stage & 1u) * s.act_elems;
    const uint16_t* act_lo = act_hi + (size_t)p.MR * Kp;
    const unsigned tag = product_tag(p, c, KIND, layer);
    const int ring = KIND == X_LM ? 0 : (layer & 1);
    stamp(c, stage, 0);
    lds_barrier();   // the XCD's slice of the stage input is in LDS
    stamp(c, stage, 1);
    const float* ssrow = (KIND == X_C || KIND == X_E) ? nullptr : s.ss0 + (stage & 1u) * 16;
    const unsigned pbit = parity_bit(c, KIND, layer, lane & 15);
    mfma_store<NSW, KTM>(p, KIND, g, c, lane, w, act_hi, act_lo, ssrow, Kp, ring, tag, pbit, 0, stage);
    stamp(c, stage, 2);
    // Loads and stores share one counter and complete out of order among each other: with stores
    // pending, "wait for the first n loads" is not expressible and every wait becomes "wait for
    // everything".  So the stores are acknowledged before any further tile is requested.
    __builtin_amdgcn_s_waitcnt(0x0f70);   // vmcnt(0)
    stamp(c, stage, 4);
    // A compute unit answers its waves' memory requests in the order they were made: what the IO waves
    // ask for behind a batch of weight tiles waits until the batch has come in (with every unit asking
    // at once, ~0.15 us per KB and wave).  So every stage requests about a fifth of a layer, in small
    // parts, here - where the unit's IO waves are between their first look at the partial sums and the
    // look that finds them.
    prefetch();
    if (KIND == X_LM) {   // further rounds of the output projection: same staged input
        for (int r = 1; r < p.lm_rounds; ++r) {
            issue_tiles<NSW, KTM>(p, g, 0, lane, w, r);
            mfma_store<NSW, KTM>(p, KIND, g, c, lane, w, act_hi, act_lo, ssrow, Kp, ring, tag, pbit, r);
        }
    }
}

// IO waves: wait for the producers of the stage input on this XCD, stage the XCD's slice in LDS, then -
// while the compute waves multiply - do the wave's reduce job of this stage.  kind is a run-time value
// (X_A .. X_LM): one copy of this code serves every product.
template <int HD>
__device__ __forceinline__ void io_stage(const XP& p, Ctx& c, const IoJobs& jb, const Lds& s, int kind, int layer, unsigned stage,
                                         f32x4& resid) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    // whose flags announce the stage input, and where it is: QKV and the output projection read x (stage E
    // of the layer before, or the prologue), Wo the attention's rows, W1|W3 x' (stage C), W2 the hidden vector
    const int wait_flag = (kind == X_A || kind == X_LM) ? F_E : kind == X_C ? F_B : kind == X_D ? F_C : F_D;
    const unsigned wait_tag = tag_of(c, (kind == X_A || kind == X_LM) ? layer - 1 : layer, wait_flag);
    const u64 region = (kind == X_A || kind == X_LM) ? p.o_a : kind == X_C ? p.o_o : kind == X_D ? p.o_x2 : p.o_h;
    const int Kp = kind == X_C ? p.KpO : kind == X_E ? p.KpH : p.KpA;
    const int nwait = wait_flag == F_E ? jb.nE : wait_flag == F_B ? jb.nB : wait_flag == F_C ? jb.nC : jb.nD;
    stamp(c, stage, 0);
    wait_flags(p, c, wait_flag, nwait, wait_tag);
    unsigned* const go = HD != 64 ? s.go : nullptr;   // every IO wave announces once per product stage
    stamp(c, stage, 1);
    // a product that follows a norm: the last IO wave adds the sums of squares up while the other three copy
    const bool normed = kind != X_C && kind != X_E;
    if (normed && wave == kCW + kNIO - 1 && lane < p.MR) {
        // The product follows a norm: the sums of squares of this XCD's slice of its input, row by row - its
        // owners' strips added in strip order - for the compute waves to send along with their partial sums.
        const int per_xcd = p.d / 16 / kXcd;
        const float* ss = reinterpret_cast<const float*>(xcd_buf(p, c.x, layer & 1) + p.o_ss) + (size_t)(kind == X_D) * per_xcd * 16 + lane;
        constexpr int NSS = HD == 64 ? 16 : 32;   // strips an XCD owns at most (all requested at once: one round trip)
        float v[NSS], a = 0.f;
#pragma unroll
        for (int i = 0; i < NSS; ++i) v[i] = i < per_xcd ? __uint_as_float(ld_u32(ss + i * 16)) : 0.f;
        announce(go);
#pragma unroll
        for (int i = 0; i < NSS; ++i) a += v[i];
        s.ss0[(stage & 1u) * 16 + lane] = a;
    }
    if (HD != 64 && kind == X_E) {   // in parts, a workgroup barrier behind each (the compute waves cross the same ones)
        const int words = Kp / 8, nparts = (p.KT[X_E][c.x] + 15) / 16;
        for (int part = 0; part < nparts; ++part) {
            stage_copy_cols(make_rsrc(p.xbuf), (unsigned)(((size_t)c.x * kRing + (layer & 1)) * p.xcd_bytes + region), p.MR, Kp,
                            s.act0 + (size_t)(stage & 1u) * s.act_elems, threadIdx.x - kCW * 64, kIOThreads, part * 64,
                            part + 1 < nparts ? part * 64 + 64 : words, part == 0 ? go : nullptr);
            if (part + 1 < nparts) lds_barrier();
        }
    } else if (!normed || wave != kCW + kNIO - 1)
        stage_copy<(HD == 64 ? 4 : 8)>(make_rsrc(p.xbuf), (unsigned)(((size_t)c.x * kRing + (layer & 1)) * p.xcd_bytes + region), p.MR, Kp,
                   s.act0 + (size_t)(stage & 1u) * s.act_elems, threadIdx.x - kCW * 64, normed ? kIOThreads - 64 : kIOThreads, go);
    stamp(c, stage, 2);
    lds_barrier();
    if (kind == X_LM) reduce_logits(p, c, wave - kCW, lane);
    else {
        reduce_job<HD>(p, c, jb, kind, layer, lane, resid, stage);
    }
    stamp(c, stage, 3);
}

// Template arguments: strips per compute wave and round / most k-tiles per XCD slice of QKV, Wo, W1|W3,
// W2; strips per wave and round of the output projection.  Weights are requested one or two stages
// ahead: Wo and W1|W3 behind QKV's products (they arrive while the attention runs), W2 and the next
// layer's QKV behind W1|W3's.
template <int NA, int KA, int NC, int KC, int ND, int KD, int NE, int KE, int NL>
__device__ __forceinline__ void compute_main(const XP& p, const Ctx& c, const Lds& s) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const GJob gA = load_gjob(p, X_A, c, wave), gC = load_gjob(p, X_C, c, wave), gD = load_gjob(p, X_D, c, wave);
    const GJob gE = load_gjob(p, X_E, c, wave), gL = load_gjob(p, X_LM, c, wave);
    v4u wA[NA * KA], wC[NC * KC], wD[ND * KD], wE[NE * KE];
    // Requests, one part per stage (see compute_stage): a buffer is refilled at the start of a stage that
    // does not use it, for its next use - QKV stage: second half of this layer's W1|W3 strips and Wo;
    // Wo stage: the next layer's QKV; W1|W3 stage: this layer's W2; W2 stage: first half of the next
    // layer's W1|W3.
    constexpr int NDh = ((ND + 1) / 2) * KD, CH = kPaceTiles;
    issue_tiles<NA, KA>(p, gA, 0, lane, wA);
    issue_tiles<ND, KD, 0, NDh>(p, gD, 0, lane, wD);
    unsigned stage = 0;
    for (int l = 0; l < p.L; ++l) {
        const u64 lb = (u64)l * p.layer_tiles;
        const bool more = l + 1 < p.L;
        compute_stage<X_A, NA, KA>(p, c, gA, s, l, stage++, p.KpA, wA, [&] {
            issue_paced<ND, KD, NDh, ND * KD, CH>(p, gD, lb, lane, wD);
            issue_paced<NC, KC, 0, NC * KC, CH>(p, gC, lb, lane, wC);
        });
        ++stage;   // attention: the IO waves' business
        compute_stage<X_C, NC, KC>(p, c, gC, s, l, stage++, p.KpO, wC, [&] {
            if (more) issue_paced<NA, KA, 0, NA * KA, CH>(p, gA, lb + p.layer_tiles, lane, wA);
        });
        compute_stage<X_D, ND, KD>(p, c, gD, s, l, stage++, p.KpA, wD, [&] { issue_paced<NE, KE, 0, NE * KE, CH>(p, gE, lb, lane, wE); });
        compute_stage<X_E, NE, KE>(p, c, gE, s, l, stage++, p.KpH, wE, [&] {
            if (more) issue_paced<ND, KD, 0, NDh, CH>(p, gD, lb + p.layer_tiles, lane, wD);
        });
    }
    v4u wL[NL * KA];
    issue_tiles<NL, KA>(p, gL, 0, lane, wL);
    compute_stage<X_LM, NL, KA>(p, c, gL, s, p.L, stage++, p.KpA, wL, [] {});
}

// ------------------------------------------------------------------------- compute waves, streamed
//
// The wide shape (d = 4096): a wave's tiles of one layer (~1.6 MB) are far more than its registers hold,
// so the weights stream through two register buffers of 16 tiles.  A stage is a list of items - (strip,
// chunk of 16 k-tiles), strips outermost - with an even count, so that an item's buffer is known at
// compile time; a buffer is refilled with the item two ahead as soon as its products are done.  Across
// a stage boundary: the next stage's first item is requested before the last item's products, its second
// when the next stage's input has been announced (see stream_stage) - more in flight during the exchange
// of activations was measured slower (the IO waves' requests queue behind it), less leaves memory idle.
// One accumulator per strip (both halves of the split activations add into it); all partial sums of a
// stage are stored at its end, behind the products, so that no store is pending while loads are waited
// for one by one.
template <int KTM, int SI, int KC>
__device__ __forceinline__ void issue_item(const XP& p, const GJob& g, u64 layer_base, int lane, v4u (&buf)[16]) {
    // A buffer resource per item whose extent is the tiles the item really has: requests beyond it (an
    // absent strip, k-tiles past the XCD's slice) come back as zeros without touching memory.
    int ns = g.ns, KT = g.KT;
    asm volatile("" : "+s"(ns), "+s"(KT));   // worked out per item, not for every item of the layer ahead of the loop
    const int have = SI < ns ? min(max(KT - KC * 16, 0), 16) : 0;
    // (the job's fields are in scalar registers - see compute_main_stream - and so is everything here)
    const char* base = reinterpret_cast<const char*>(p.wpack) + (layer_base + g.tile0 + (u64)SI * KT + KC * 16) * 1024;
#pragma unroll
    for (int q = 0; q < 4; ++q) {   // four tiles per resource: their offsets fit the instruction's immediate field
        if (KC * 16 + q * 4 < KTM) {
            const rsrc_t r = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(base + q * 4096), 0, max(have - q * 4, 0) * 1024, 0x00020000);
#pragma unroll
            for (int kt = q * 4; kt < q * 4 + 4; ++kt)
                if (KC * 16 + kt < KTM) buf[kt] = __builtin_amdgcn_raw_buffer_load_b128(r, (unsigned)lane * 16u + (kt - q * 4) * 1024u, 0, kNonTemporal);
        }
    }
}

// The first item of the stage that follows, for the stage before it to request.
template <int KTM>
struct NextItem {
    const XP& p; const GJob& g; u64 lb; int lane;
    __device__ __forceinline__ void operator()(v4u (&b)[16]) const { issue_item<KTM, 0, 0>(p, g, lb, lane, b); }
};

// Items IT, IT + 1, .. of a stage of NS strips x NKC chunks; cur holds item IT, nxt item IT + 1.
template <int NS, int NKC, int KTM, int IT, bool PARTS, class Next>
__device__ __forceinline__ void stream_items(const XP& p, const GJob& g, u64 layer_base, int lane, const uint16_t* act_hi,
                                             const uint16_t* act_lo, v4u (&cur)[16], v4u (&nxt)[16], f32x4 (&acc)[NS], Next&& next) {
    if constexpr (IT < NS * NKC) {
        constexpr int si = IT / NKC, kc = IT % NKC;
        if (PARTS && IT > 0 && IT < NKC) lds_barrier();   // the input's next chunk of 16 k-tiles is in LDS
#pragma unroll
        for (int kt = 0; kt < 16; ++kt) {
            if (kc * 16 + kt < KTM) {
                const bf16x8 h = __builtin_bit_cast(bf16x8, *reinterpret_cast<const v4u*>(act_hi + (kc * 16 + kt) * 32));
                const bf16x8 l = __builtin_bit_cast(bf16x8, *reinterpret_cast<const v4u*>(act_lo + (kc * 16 + kt) * 32));
                const bf16x8 a = __builtin_bit_cast(bf16x8, cur[kt]);
                acc[si] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, h, acc[si], 0, 0, 0);
                acc[si] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, l, acc[si], 0, 0, 0);
            }
        }
        if constexpr (IT + 2 < NS * NKC) {   // the freed buffer takes the item two ahead
            issue_item<KTM, (IT + 2) / NKC, (IT + 2) % NKC>(p, g, layer_base, lane, cur);
            stream_items<NS, NKC, KTM, IT + 1, PARTS>(p, g, layer_base, lane, act_hi, act_lo, nxt, cur, acc, next);
        } else if constexpr (IT + 2 == NS * NKC) {
            next(cur);   // first item of the next stage
            stream_items<NS, NKC, KTM, IT + 1, PARTS>(p, g, layer_base, lane, act_hi, act_lo, nxt, cur, acc, next);
        }
    }
}

// One product stage of the streamed kind.  On entry b0 holds (or is about to receive) item 0; next(buf) requests
// the first item of the following stage into buf.
template <int KIND, int NS, int NKC, int KTM, class Next>
__device__ __forceinline__ void stream_stage(const XP& p, const Ctx& c, const GJob& g, const Lds& s, int layer, unsigned stage, int Kp,
                                             u64 layer_base, v4u (&b0)[16], v4u (&b1)[16], Next&& next) {
    static_assert((NS * NKC) % 2 == 0 && NS * NKC >= 2, "a stage has an even number of items");
    int lane = threadIdx.x & 63;
    asm volatile("" : "+v"(lane));   // what depends on the lane is worked out again in every stage: kept across the
                                     // layer loop for all stages at once it would not fit the registers next to the tiles
    const int col = lane & 15, kg = lane >> 4;
    const uint16_t* act_hi = s.act0 + (size_t)(stage & 1u) * s.act_elems + (size_t)(col < p.MR ? col : 0) * Kp + kg * 8;
    const uint16_t* act_lo = act_hi + (size_t)p.MR * Kp;
    const unsigned tag = product_tag(p, c, KIND, layer);
    const int ring = KIND == X_LM ? 0 : (layer & 1);
    const unsigned pbit = parity_bit(c, KIND, layer, col);
    f32x4 acc[NS];
#pragma unroll
    for (int i = 0; i < NS; ++i) acc[i] = (f32x4){0.f, 0.f, 0.f, 0.f};
    stamp(c, stage, 0);
    // The second item is requested when all four IO waves have made their first requests for the stage input (they
    // count themselves in LDS, see announce): the unit answers requests in order, so the item comes in behind
    // the input and is on its way while the input goes to LDS.  Earlier, it would hold up what the IO waves ask
    // for on the way there; behind the barrier, its whole latency would be exposed.  Only a hint: the wait is
    // short and bounded, and running out of it changes nothing but the timing.
    // (Wo's two items are both requested at once: the attention runs in between, and they are in long before its
    // output is staged.)
    const unsigned l5 = stage / 5u, st5 = stage - 5u * l5;                        // (stage = 5 layer + 0, 2, 3, 4; the output projection 5 L)
    const unsigned want = 4u * (4u * l5 + (st5 ? st5 - 1u : 0u) + 1u);           // four announcements per product stage so far
    for (unsigned spins = 0; KIND != X_C && spins < 8192u; ++spins) {
        if ((int)(__hip_atomic_load(s.go, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) - want) >= 0) break;
        __builtin_amdgcn_s_sleep(1);
    }
    issue_item<KTM, 1 / NKC, 1 % NKC>(p, g, layer_base, lane, b1);
    lds_barrier();   // the XCD's slice of the stage input is in LDS
    stamp(c, stage, 1);
    stream_items<NS, NKC, KTM, 0, (KIND == X_E && NKC > 1)>(p, g, layer_base, lane, act_hi, act_lo, b0, b1, acc, next);
    if (c.dbg) {
        asm volatile("" :: "v"(acc[NS - 1]));
        stamp(c, stage, 3);
    }
    if (KIND != X_C && KIND != X_E && kg == 0 && col < p.MR && g.ns > 0)   // this XCD's share of the rows' sums of squares rides along
        st_tagged(p.pss[KIND] + ((((size_t)ring * kXcd + c.x) * kPer + c.j) * kCW + (threadIdx.x >> 6)) * 32 + col,
                  s.ss0[(stage & 1u) * 16 + col], tag);
    const rsrc_t out = make_rsrc(p.part[KIND]);
    const unsigned at8 = (unsigned)((((size_t)ring * kXcd + c.x) * p.nstrips[KIND] + g.s0) * 16 + col) * 64u + kg * 16u;
#pragma unroll
    for (int si = 0; si < NS; ++si) {
        const f32x4 v = acc[si];
        if (si < g.ns && col < p.MR)
            st_16(out, at8 + si * 1024u, (v4u){(__float_as_uint(v[0]) & ~1u) | pbit, (__float_as_uint(v[1]) & ~1u) | pbit,
                                               (__float_as_uint(v[2]) & ~1u) | pbit, (__float_as_uint(v[3]) & ~1u) | pbit});
    }
    stamp(c, stage, 2);
    stamp(c, stage, 4);
}

// Template arguments: strips per compute wave of QKV, Wo, W1|W3 (rounded up to even), W2, the output
// projection; k-tiles of an XCD's slice of the hidden vector (the other slices have 16).
template <int NA, int NC, int ND, int NE, int KE, int NL>
__device__ __forceinline__ void compute_main_stream(const XP& p, const Ctx& c, const Lds& s) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    auto job = [&](int kind) {   // the same in every lane: kept in scalar registers
        GJob g = load_gjob(p, kind, c, wave);
        g.s0 = __builtin_amdgcn_readfirstlane(g.s0); g.ns = __builtin_amdgcn_readfirstlane(g.ns); g.KT = __builtin_amdgcn_readfirstlane(g.KT);
        g.tile0 = uniform64(g.tile0);
        return g;
    };
    const GJob gA = job(X_A), gC = job(X_C), gD = job(X_D), gE = job(X_E), gL = job(X_LM);
    constexpr int NKE = (KE + 15) / 16;
    v4u b0[16], b1[16];
    issue_item<16, 0, 0>(p, gA, 0, lane, b0);
    unsigned stage = 0;
    for (int l = 0; l < p.L; ++l) {
        const u64 lb = (u64)l * p.layer_tiles;
        const bool more = l + 1 < p.L;
        stream_stage<X_A, NA, 1, 16>(p, c, gA, s, l, stage++, p.KpA, lb, b0, b1, NextItem<16>{p, gC, lb, lane});
        ++stage;   // attention: the IO waves' business
        stream_stage<X_C, NC, 1, 16>(p, c, gC, s, l, stage++, p.KpO, lb, b0, b1, NextItem<16>{p, gD, lb, lane});
        stream_stage<X_D, ND, 1, 16>(p, c, gD, s, l, stage++, p.KpA, lb, b0, b1, NextItem<KE>{p, gE, lb, lane});
        // (the output projection's tiles follow the layers in the stream; it has no more strips per wave than QKV)
        stream_stage<X_E, NE, NKE, KE>(p, c, gE, s, l, stage++, p.KpH, lb, b0, b1,
                                       NextItem<16>{p, more ? gA : gL, more ? lb + p.layer_tiles : 0, lane});
    }
    const GJob none = {0, 0, 0, 0};
    stream_stage<X_LM, NL, 1, 16>(p, c, gL, s, p.L, stage++, p.KpA, 0, b0, b1, NextItem<16>{p, none, 0, lane});
}

template <int RPJ, int HD>
__device__ __forceinline__ void io_main(const XP& p, Ctx& c, const Lds& s) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const IoJobs jb = load_io_jobs<HD>(p, c, wave - kCW, lane);
    f32x4 resid = (f32x4){0.f, 0.f, 0.f, 0.f};   // the wave's strip of the residual stream (owners of Wo / W2 strips)
    if (jb.sE >= 0) {   // Prologue: the owners of the residual strips pick their slice of the embedded rows up
                                // and publish it as stage E of "layer -1" would.
        const int strip = jb.sE, col = lane & 15, quad = lane >> 4;
        const uint2 gain = *reinterpret_cast<const uint2*>(p.blob + p.g1_off / 2 + strip * 16 + 4 * quad);
        resid = col < p.MR ? *reinterpret_cast<const f32x4*>(p.X + (size_t)col * p.d + strip * 16 + 4 * quad)
                           : (f32x4){0.f, 0.f, 0.f, 0.f};
        put_stream(p, c, 0, 0, strip, lane, resid, gain);
        raise_flag(p, c, F_E, jb.tE, tag_of(c, -1, F_E));
    }
    unsigned joins = 0;
    // stages of the pass in order: per layer QKV, attention, Wo, W1|W3, W2; then the output projection
    // on the final norm's input (published by the last stage E into ring slot L & 1)
    const unsigned nstages = 5u * (unsigned)p.L + 1u;
#pragma nounroll
    for (unsigned stage = 0; stage < nstages; ++stage) {
        const int l = (int)(stage / 5u), st = (int)(stage - 5u * (unsigned)l);
        if (st == 1) attn_io<RPJ, HD>(p, c, jb, s, l, stage, joins);
        else io_stage<HD>(p, c, jb, s, l == p.L ? X_LM : st == 0 ? X_A : st == 2 ? X_C : st == 3 ? X_D : X_E, l, stage, resid);
    }
}

template <int NA, int KA, int NC, int KC, int ND, int KD, int NE, int KE, int NL, int RPJ, int HD = 64>
__global__ __launch_bounds__(kThreads, 1) void verify_xcd_kernel(const XP* __restrict__ params, unsigned epoch0, unsigned par, unsigned par_lm, u64* dbg) {
    // The parameter block lives in device memory (written when the step shape changes): tables in it are
    // indexed with run-time values, which a by-value kernel argument would answer with a private copy.
    const XP& p = *params;
    extern __shared__ uint4 smem_raw[];
    Lds s;
    const size_t act_elems = (size_t)2 * p.MR * max(max(p.KpA, p.KpO), p.KpH);
    s.join = reinterpret_cast<unsigned*>(smem_raw);
    s.go = s.join + 1;
    s.act0 = reinterpret_cast<uint16_t*>(smem_raw + 1);
    s.act_elems = (unsigned)act_elems;
    s.part = reinterpret_cast<float*>(s.act0 + 2 * act_elems);
    s.qs = s.part + kNIO * RPJ * (HD + 4);
    s.ss0 = s.qs + RPJ * HD;
    if (threadIdx.x == 0) { *s.join = 0u; *s.go = 0u; }
    __syncthreads();
    Ctx c;
    c.x = blockIdx.x % kXcd; c.j = blockIdx.x / kXcd; c.epoch0 = epoch0; c.par = par; c.par_lm = par_lm; c.dead = false; c.err = p.err; c.dbg = dbg;
    if (xcc_id() != c.x) give_up(c);   // the dispatch order this layout relies on does not hold: fail, never hang
    // The two kinds of waves run separate code (and cross the same workgroup barriers), so that neither
    // carries the other's registers: compute waves the weights in flight, IO waves the attention's keys
    // and values and the partial sums of a reduce job.
    if ((threadIdx.x >> 6) >= kCW) io_main<RPJ, HD>(p, c, s);
    else compute_main<NA, KA, NC, KC, ND, KD, NE, KE, NL>(p, c, s);
}

// The same pass for the wide shape: the compute waves stream their tiles (see compute_main_stream).
template <int NA, int NC, int ND, int NE, int KE, int NL, int RPJ, int HD>
__global__ __launch_bounds__(kThreads, 1) void verify_xcd_stream_kernel(const XP* __restrict__ params, unsigned epoch0, unsigned par, unsigned par_lm,
                                                                        u64* dbg) {
    const XP& p = *params;
    extern __shared__ uint4 smem_raw[];
    Lds s;
    const size_t act_elems = (size_t)2 * p.MR * max(max(p.KpA, p.KpO), p.KpH);
    s.join = reinterpret_cast<unsigned*>(smem_raw);
    s.go = s.join + 1;
    s.act0 = reinterpret_cast<uint16_t*>(smem_raw + 1);
    s.act_elems = (unsigned)act_elems;
    s.part = reinterpret_cast<float*>(s.act0 + 2 * act_elems);
    s.qs = s.part + kNIO * RPJ * (HD + 4);
    s.ss0 = s.qs + RPJ * HD;
    if (threadIdx.x == 0) { *s.join = 0u; *s.go = 0u; }
    __syncthreads();
    Ctx c;
    c.x = blockIdx.x % kXcd; c.j = blockIdx.x / kXcd; c.epoch0 = epoch0; c.par = par; c.par_lm = par_lm; c.dead = false; c.err = p.err; c.dbg = dbg;
    if (xcc_id() != c.x) give_up(c);
    if ((threadIdx.x >> 6) >= kCW) io_main<RPJ, HD>(p, c, s);
    else compute_main_stream<NA, NC, ND, NE, KE, NL>(p, c, s);
}

// Copies one matrix into the packed order: tile T of the stream is (strip, k-tile) = desc[T]; lane l
// holds row l % 16, columns 8 * (l / 16) .. + 7 of that tile.  pairs > 0: W1 | W3 with strip rows 0..7
// from W1 and 8..15 from W3 (pairs = rows of W1).
__global__ void xcd_repack_kernel(const uint16_t* W, int K, int pairs, int row0, const uint32_t* desc, uint4* out) {
    const size_t tile = blockIdx.x;
    const int lane = threadIdx.x;
    const uint32_t dsc = desc[tile];
    const int strip = dsc >> 12, kt = dsc & 4095, r = lane & 15;
    size_t row = (size_t)(row0 + strip * 16 + r);
    if (pairs > 0) row = (size_t)((r < 8 ? 0 : pairs) + strip * 8 + (r & 7));
    const size_t col = (size_t)kt * 32 + (lane >> 4) * 8;
    out[tile * 64 + lane] = *reinterpret_cast<const uint4*>(W + row * K + col);
}

size_t up256(size_t x) { return (x + 255) & ~(size_t)255; }

}  // namespace

// ------------------------------------------------------------------------- host: plan

struct XcdPlan {
    bool ok;
    int KT[X_NK][kXcd], kt0[X_NK][kXcd], nstrips[X_NK];
    int hd0[kXcd + 1], ke0[kXcd + 1];
    size_t xbase[X_NK][kXcd], layer_tiles, total_tiles;
    int njobs[F_NF][kXcd];
    int NSW[X_NK];                 // strips per compute wave and round the plan needs
    int lm_rounds;
    int KpA, KpO, KpH;
    unsigned par, par_lm;          // parities of the partial-sum words (see parity_bit), per row
    std::vector<int16_t> gtab, rtab, ptab;
    int poff[X_NK];
    std::vector<uint8_t> params;   // the parameter block as last uploaded
    std::vector<uint32_t> desc;    // (strip << 12) | k-tile per packed tile, kinds in stream order of one layer, then the output projection
    size_t desc_kind[X_NK][kXcd];  // index of (kind, XCD)'s first descriptor
    unsigned epoch;
};

namespace {

bool xcd_shape_ok(const hawk_ctx* c) {
    if (c->cfg.dtype != HAWK_BF16) return false;
    if (!((c->d == 1280 && c->m == 3456 && c->H == 20 && c->hd == 64) || (c->d == 768 && c->m == 2048 && c->H == 12 && c->hd == 64) ||
          (c->d == 4096 && c->m == 11008 && c->H == 32 && c->hd == 128)))
        return false;
    if (c->Vs % (16 * kXcd) || c->d % (32 * kXcd) || c->H < kXcd) return false;
    return true;
}

// Contiguous split of n items into `parts` ranges; the first `n % parts` ranges (or the last, if
// extra_last) take one more.
void split_ranges(int n, int parts, bool extra_last, std::vector<int>& start) {
    start.assign(parts + 1, 0);
    const int base = n / parts, extra = n % parts;
    for (int i = 0; i < parts; ++i) {
        const bool more = extra_last ? i >= parts - extra : i < extra;
        start[i + 1] = start[i] + base + (more ? 1 : 0);
    }
}

void build_xcd_plan(const hawk_ctx* c, XcdPlan* P) {
    P->ok = xcd_shape_ok(c);
    P->epoch = 0;
    P->par = P->par_lm = 0;   // the areas are cleared below: parity 0 everywhere
    if (!P->ok) return;
    const int d = c->d, m = c->m, H = c->H;
    P->nstrips[X_A] = 3 * d / 16; P->nstrips[X_C] = d / 16; P->nstrips[X_D] = 2 * m / 16; P->nstrips[X_E] = d / 16;
    P->nstrips[X_LM] = c->Vs / 16;
    std::vector<int> hs, es;
    split_ranges(H, kXcd, false, hs);           // heads per XCD
    split_ranges(m / 32, kXcd, false, es);      // k-tiles of the MLP's hidden vector per XCD
    for (int x = 0; x <= kXcd; ++x) { P->hd0[x] = hs[x]; P->ke0[x] = es[x]; }
    int maxO = 0, maxH = 0;
    for (int x = 0; x < kXcd; ++x) {
        P->KT[X_A][x] = P->KT[X_D][x] = P->KT[X_LM][x] = d / 32 / kXcd;
        P->kt0[X_A][x] = P->kt0[X_D][x] = P->kt0[X_LM][x] = x * (d / 32 / kXcd);
        P->KT[X_C][x] = (c->hd / 32) * (hs[x + 1] - hs[x]); P->kt0[X_C][x] = (c->hd / 32) * hs[x];
        P->KT[X_E][x] = es[x + 1] - es[x]; P->kt0[X_E][x] = es[x];
        maxO = std::max(maxO, P->KT[X_C][x] * 32);
        maxH = std::max(maxH, P->KT[X_E][x] * 32);
    }
    P->KpA = d / kXcd + 8; P->KpO = maxO + 8; P->KpH = maxH + 8;
    // strips of (unit j, compute wave w): contiguous; the kinds alternate which half of the units takes
    // the extra strip so that every unit streams about the same bytes per layer
    P->gtab.assign((size_t)X_NK * kPer * kCW * 2, 0);
    for (int k = 0; k < X_NK; ++k) {
        std::vector<int> us, ws;
        split_ranges(P->nstrips[k], kPer, k == X_A || k == X_D, us);
        int need = 0;
        for (int j = 0; j < kPer; ++j) {
            split_ranges(us[j + 1] - us[j], kCW, false, ws);
            for (int w = 0; w < kCW; ++w) {
                P->gtab[(((size_t)k * kPer + j) * kCW + w) * 2] = (int16_t)(us[j] + ws[w]);
                P->gtab[(((size_t)k * kPer + j) * kCW + w) * 2 + 1] = (int16_t)(ws[w + 1] - ws[w]);
                need = std::max(need, ws[w + 1] - ws[w]);
            }
        }
        P->NSW[k] = need;
        if (P->nstrips[k] > 32767) P->ok = false;
    }
    for (int k = 0; k < X_NK; ++k) {   // producer of every strip (the output projection takes two rounds of half the strips)
        P->poff[k] = (int)P->ptab.size();
        P->ptab.resize(P->ptab.size() + P->nstrips[k], 0);
        const int per_round = k == X_LM ? 4 : P->NSW[k];   // the kernel's instances take 4 output-projection strips per round
        for (int j = 0; j < kPer; ++j)
            for (int w = 0; w < kCW; ++w) {
                const int16_t* g = &P->gtab[(((size_t)k * kPer + j) * kCW + w) * 2];
                for (int i = 0; i < g[1]; ++i)
                    P->ptab[P->poff[k] + g[0] + i] = (int16_t)((j * kCW + w) * 2 + std::min(i / std::max(per_round, 1), 1));
            }
    }
    // packed stream of a layer: per kind, per XCD, strips in order, the XCD's k-tiles of each
    P->desc.clear();
    size_t off = 0;
    for (int k = 0; k < X_NK; ++k) {
        if (k == X_LM) P->layer_tiles = off;
        for (int x = 0; x < kXcd; ++x) {
            P->xbase[k][x] = k == X_LM ? (size_t)c->L * P->layer_tiles + (off - P->layer_tiles) : off;
            P->desc_kind[k][x] = P->desc.size();
            for (int s = 0; s < P->nstrips[k]; ++s)
                for (int t = 0; t < P->KT[k][x]; ++t) P->desc.push_back(((uint32_t)s << 12) | (uint32_t)(P->kt0[k][x] + t));
            off += (size_t)P->nstrips[k] * P->KT[k][x];
        }
    }
    P->total_tiles = (size_t)c->L * P->layer_tiles + (off - P->layer_tiles);
    // reduce jobs: the IO wave (unit, wave) of the owner XCD that finishes a strip, and its flag slot
    P->rtab.assign((size_t)X_NK * kXcd * kPer * kNIO * 3, -1);
    for (int f = 0; f < F_NF; ++f)
        for (int x = 0; x < kXcd; ++x) P->njobs[f][x] = 0;
    auto owner_of = [&](int k, int s) -> int {
        if (k == X_A) {   // the XCD that owns the strip's head
            const int h = ((s * 16) % d) / c->hd;
            for (int x = 0; x < kXcd; ++x)
                if (h < hs[x + 1]) return x;
        }
        if (k == X_C || k == X_E) return s / (d / 16 / kXcd);
        if (k == X_D) {   // the XCD that owns the k-tile of the hidden vector the strip's 8 values fall into
            const int t = (s * 8) / 32;
            for (int x = 0; x < kXcd; ++x)
                if (t < es[x + 1]) return x;
        }
        return 0;
    };
    const int flag_of[4] = {F_A, F_C, F_D, F_E};
    for (int k = X_A; k <= X_E; ++k) {
        int count[kXcd] = {0}, total[kXcd] = {0};
        for (int s = 0; s < P->nstrips[k]; ++s) total[owner_of(k, s)]++;
        for (int s = 0; s < P->nstrips[k]; ++s) {
            const int x = owner_of(k, s), i = count[x]++;
            // Wo and W2 strips: the same wave owns the strip's residual in both (last IO wave of unit i).
            // QKV strips: the last units of the XCD, three waves each - the first units run the attention
            // jobs and should start on their keys and values at once.  W1|W3 strips go round the units.
            const int nu = (total[x] + kNIO - 2) / (kNIO - 1);
            const int slots_d = kPer * (kNIO - 1);   // W1|W3: IO waves 0 .. 2 of every unit; beyond that a wave takes a second strip
            const bool second = k == X_D && i >= slots_d;
            const int id = second ? i - slots_d : i;
            const int j = (k == X_C || k == X_E) ? i : k == X_A ? kPer - 1 - i % nu : id % kPer;
            const int w = (k == X_C || k == X_E) ? kNIO - 1 : k == X_A ? i / nu : id / kPer;
            if (j >= kPer || w >= ((k == X_C || k == X_E) ? kNIO : kNIO - 1) || id >= kMaxJobs) { P->ok = false; return; }
            int16_t* e = &P->rtab[((((size_t)k * kXcd + x) * kPer + j) * kNIO + w) * 3];
            if (second) {
                e[2] = (int16_t)s;
            } else {
                e[0] = (int16_t)s;
                e[1] = (int16_t)i;
            }
        }
        for (int x = 0; x < kXcd; ++x) P->njobs[flag_of[k]][x] = k == X_D ? std::min(count[x], kPer * (kNIO - 1)) : count[x];
    }
    const int per_round = kPer * kCW * P->NSW[X_LM];
    (void)per_round;
    P->lm_rounds = 1;
}

// Attention jobs of a step with RS rows per sequence: (sequence, head, row group) per unit of the XCD
// that owns the head.
bool attn_jobs(const hawk_ctx* c, const XcdPlan* P, int RS, int* RPJ, std::vector<int16_t>& atab, int (&nj)[kXcd]) {
    int rpj = 1;
    for (;; ++rpj) {
        if (rpj > 2) return false;
        bool fits = true;
        for (int x = 0; x < kXcd; ++x)
            fits = fits && (P->hd0[x + 1] - P->hd0[x]) * c->S * ((RS + rpj - 1) / rpj) <= kPer;
        if (fits) break;
    }
    *RPJ = rpj;
    atab.assign((size_t)kXcd * kPer * 4, -1);
    for (int x = 0; x < kXcd; ++x) {
        int i = 0;
        for (int seq = 0; seq < c->S; ++seq)
            for (int h = P->hd0[x]; h < P->hd0[x + 1]; ++h)
                for (int rg = 0; rg < (RS + rpj - 1) / rpj; ++rg, ++i) {
                    int16_t* e = &atab[((size_t)x * kPer + i) * 4];
                    e[0] = (int16_t)seq; e[1] = (int16_t)h; e[2] = (int16_t)rg; e[3] = (int16_t)i;
                }
        nj[x] = i;
    }
    return true;
}

// Regions of one XCD buffer (bytes): split planes are uint16 [2][16][Kp].
size_t xcd_buf_layout(const XcdPlan* P, XP* p) {
    size_t at = 0;
    auto take = [&](size_t n) { size_t a = at; at = up256(at + n); return a; };
    const size_t a = take((size_t)2 * 16 * P->KpA * 2), q = take((size_t)16 * (P->KpO - 8) * 8);   // queries: {value, tag}
    const size_t kv = take((size_t)2 * 16 * ((P->KpO - 8) / 64) * 16 * 16);   // appended keys | values: [2][16 rows][heads][16 words] {fp16 pair, tag} x 2
    const size_t o = take((size_t)2 * 16 * P->KpO * 2), x2 = take((size_t)2 * 16 * P->KpA * 2);
    const size_t h = take((size_t)2 * 16 * P->KpH * 2);
    const size_t ss = take((size_t)2 * 32 * 16 * 4);   // sums of squares of the XCD's strips: [2][strips of an XCD <= 32][16 rows]
    if (p) { p->o_a = a; p->o_q = q; p->o_kv = kv; p->o_o = o; p->o_x2 = x2; p->o_h = h; p->o_ss = ss; }
    return at;
}

}  // namespace

size_t xcd_workspace(const hawk_ctx* c, size_t base, XcdOffsets* o) {
    memset(o, 0, sizeof *o);
    XcdPlan P;
    build_xcd_plan(c, &P);
    if (!P.ok) return 0;
    size_t p = base;
    auto take = [&](size_t bytes) { size_t at = p; p = up256(p + bytes); return at; };
    o->wpack = take(P.total_tiles * 1024);
    o->zero = take(1024);
    o->desc = take(P.desc.size() * 4);
    o->gtab = take(P.gtab.size() * 2);
    o->rtab = take(P.rtab.size() * 2);
    o->ptab = take(P.ptab.size() * 2);
    o->atab = take((size_t)kXcd * kPer * 4 * 2);
    o->xp = take(4096);
    for (int k = 0; k < X_NK; ++k)
        o->part[k] = take((size_t)(k == X_LM ? 1 : kRing) * kXcd * P.nstrips[k] * 16 * 16 * 4);
    for (int k = 0; k < X_NK; ++k)
        o->pss[k] = (k == X_C || k == X_E) ? 0 : take((size_t)kRing * kXcd * kPer * kCW * 2 * 16 * 8);
    o->xcd_bytes = xcd_buf_layout(&P, nullptr);
    o->xbuf = take((size_t)kXcd * kRing * o->xcd_bytes);
    o->lflag = take((size_t)kXcd * F_NF * kMaxJobs * 4);
    o->dbg = take((size_t)2 * 512 * 16 * 8);
    o->err = take(256);
    o->rope = take((size_t)c->Tmax * (c->hd / 2) * 8);
    return p - base;
}

XcdPlan* xcd_create(hawk_ctx* c) {
    XcdPlan* P = new XcdPlan();
    build_xcd_plan(c, P);
    if (!P->ok) return P;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
        cus != kNWG) {   // the layout needs exactly one workgroup per unit, 32 units per XCD
        P->ok = false;
        return P;
    }
    const XcdOffsets& o = c->xoff;
    bool good = true;
    good = good && hipMemcpyAsync(c->ws + o.desc, P->desc.data(), P->desc.size() * 4, hipMemcpyHostToDevice, c->stream) == hipSuccess;
    good = good && hipMemcpyAsync(c->ws + o.gtab, P->gtab.data(), P->gtab.size() * 2, hipMemcpyHostToDevice, c->stream) == hipSuccess;
    good = good && hipMemcpyAsync(c->ws + o.rtab, P->rtab.data(), P->rtab.size() * 2, hipMemcpyHostToDevice, c->stream) == hipSuccess;
    good = good && hipMemcpyAsync(c->ws + o.ptab, P->ptab.data(), P->ptab.size() * 2, hipMemcpyHostToDevice, c->stream) == hipSuccess;
    // tags start at 1: zeroed flag words, partial sums and sums of squares are "older than everything"
    good = good && hipMemsetAsync(c->ws + o.zero, 0, 1024, c->stream) == hipSuccess;
    good = good && hipMemsetAsync(c->ws + o.lflag, 0, (size_t)kXcd * F_NF * kMaxJobs * 4, c->stream) == hipSuccess;
    for (int k = 0; k < X_NK; ++k)
        good = good && hipMemsetAsync(c->ws + o.part[k], 0, (size_t)(k == X_LM ? 1 : kRing) * kXcd * P->nstrips[k] * 16 * 16 * 4,
                                      c->stream) == hipSuccess;
    for (int k = 0; k < X_NK; ++k)
        if (k != X_C && k != X_E)
            good = good && hipMemsetAsync(c->ws + o.pss[k], 0, (size_t)kRing * kXcd * kPer * kCW * 2 * 16 * 8, c->stream) == hipSuccess;
    good = good && hipMemsetAsync(c->ws + o.xbuf, 0, (size_t)kXcd * kRing * o.xcd_bytes, c->stream) == hipSuccess;
    if (!c->err_ready) {   // no streaming plan set them up (a shape only this layout takes): own error word and rotary table
        std::vector<float> rope((size_t)c->Tmax * (c->hd / 2) * 2);
        for (int pos = 0; pos < c->Tmax; ++pos)
            for (int j = 0; j < c->hd / 2; ++j) {
                const double ang = (double)pos * pow((double)c->cfg.rope_theta, -2.0 * j / (double)c->hd);
                rope[((size_t)pos * (c->hd / 2) + j) * 2] = (float)cos(ang);
                rope[((size_t)pos * (c->hd / 2) + j) * 2 + 1] = (float)sin(ang);
            }
        good = good && hipMemsetAsync(c->ws + o.err, 0, 256, c->stream) == hipSuccess;
        good = good && hipMemcpyAsync(c->ws + o.rope, rope.data(), rope.size() * 4, hipMemcpyHostToDevice, c->stream) == hipSuccess;
        good = good && hipStreamSynchronize(c->stream) == hipSuccess;   // the table is a local
        if (good) { c->err_off = o.err; c->rope_off = o.rope; c->err_ready = 1; }
    }
    good = good && hipStreamSynchronize(c->stream) == hipSuccess;
    if (!good) P->ok = false;
    return P;
}

void xcd_destroy(XcdPlan* P) { delete P; }

// Re-tiles every matrix of the loaded blob into the packed order (after hawk_load).
int xcd_repack(hawk_ctx* c) {
    XcdPlan* P = c->xplan;
    if (!P || !P->ok) return 0;
    const uint16_t* blob = wsp<uint16_t>(c, c->off.blob);
    uint4* wp = wsp<uint4>(c, c->xoff.wpack);
    const uint32_t* desc = wsp<uint32_t>(c, c->xoff.desc);
    auto run = [&](size_t blob_off, int K, int kind, size_t layer_base, int pairs, int row0) {
        for (int x = 0; x < kXcd; ++x) {
            const size_t tiles = (size_t)P->nstrips[kind] * P->KT[kind][x];
            xcd_repack_kernel<<<(unsigned)tiles, 64, 0, c->stream>>>(blob + blob_off / 2, K, pairs, row0, desc + P->desc_kind[kind][x],
                                                                    wp + (layer_base + P->xbase[kind][x]) * 64);
        }
    };
    for (int l = 0; l < c->L; ++l) {
        const size_t lb = (size_t)l * P->layer_tiles;
        run(c->w.Wqkv[l], c->d, X_A, lb, 0, 0);
        run(c->w.Wo[l], c->d, X_C, lb, 0, 0);
        run(c->w.W13[l], c->d, X_D, lb, c->m, 0);
        run(c->w.W2[l], c->m, X_E, lb, 0, 0);
    }
    run(c->w.W_out, c->d, X_LM, 0, 0, c->cfg.samp_lo);
    if (hipGetLastError() != hipSuccess) return -1;
    return hipStreamSynchronize(c->stream) == hipSuccess ? 0 : -1;
}

namespace {

struct XcdShape { int NA, KA, NC, KC, ND, KD, NE, KE, NL; };

size_t xcd_lds_bytes(const hawk_ctx* c, const XcdPlan* P, int RPJ, int MR) {
    const size_t act = (size_t)2 * MR * std::max(std::max(P->KpA, P->KpO), P->KpH) * 2;   // two planes of the rows in flight
    return 16 + 2 * act + (size_t)(kNIO * RPJ * (c->hd + 4) + RPJ * c->hd + 32) * 4 + 64;
}

}  // namespace

bool xcd_ok(const hawk_ctx* c, int k) {
    const XcdPlan* P = c->xplan;
    if (!P || !P->ok || c->path != 1 || !stream_has_err_word(c)) return false;   // (error word and rotary table: the streaming plan's)
    const int RS = k + 1, MR = c->S * RS;
    if (MR > 16) return false;
    for (int x = 0; x < kXcd; ++x)
        if ((P->hd0[x + 1] - P->hd0[x]) * c->S * ((RS + 1) / 2) > kPer) return false;
    if (xcd_lds_bytes(c, P, 2, MR) > (size_t)160 * 1024) return false;
    return true;
}

int launch_verify_xcd(hawk_ctx* c, int k, const int32_t* tree_depth, const unsigned long long* tree_anc) {
    XcdPlan* P = c->xplan;
    XP p;
    memset(&p, 0, sizeof p);
    const XcdOffsets& o = c->xoff;
    const int RS = k + 1;
    std::vector<int16_t> atab;
    int nattn[kXcd], RPJ = 1;
    if (!attn_jobs(c, P, RS, &RPJ, atab, nattn)) return -1;
    p.wpack = wsp<uint4>(c, o.wpack);
    p.zero_tile = wsp<uint4>(c, o.zero);
    p.layer_tiles = P->layer_tiles;
    for (int kk = 0; kk < X_NK; ++kk) {
        p.nstrips[kk] = P->nstrips[kk];
        p.part[kk] = wsp<u64>(c, o.part[kk]);
        for (int x = 0; x < kXcd; ++x) { p.xbase[kk][x] = P->xbase[kk][x]; p.KT[kk][x] = P->KT[kk][x]; }
    }
    for (int x = 0; x <= kXcd; ++x) { p.hd0[x] = P->hd0[x]; p.ke0[x] = P->ke0[x]; }
    for (int f = 0; f < F_NF; ++f)
        for (int x = 0; x < kXcd; ++x) p.njobs[f][x] = f == F_B ? nattn[x] : P->njobs[f][x];
    p.gtab = wsp<int16_t>(c, o.gtab); p.rtab = wsp<int16_t>(c, o.rtab); p.ptab = wsp<int16_t>(c, o.ptab);
    for (int k = 0; k < X_NK; ++k) p.poff[k] = P->poff[k]; p.atab = wsp<int16_t>(c, o.atab);
    for (int kk = 0; kk < X_NK; ++kk) p.pss[kk] = (kk == X_C || kk == X_E) ? nullptr : wsp<u64>(c, o.pss[kk]);
    p.xbuf = c->ws + o.xbuf; p.xcd_bytes = o.xcd_bytes;
    (void)xcd_buf_layout(P, &p);
    p.lflag = wsp<unsigned>(c, o.lflag);
    p.blob = wsp<uint16_t>(c, c->off.blob);
    p.g1_off = c->w.g1[0]; p.g2_off = c->w.g2[0];
    p.layer_bytes = c->L > 1 ? c->w.g1[1] - c->w.g1[0] : 0;
    p.gf_off = c->w.g_f;
    p.rope = wsp<float2>(c, c->rope_off);
    p.Kc = wsp<_Float16>(c, c->off.kc); p.Vc = wsp<_Float16>(c, c->off.vc);
    p.X = wsp<float>(c, c->off.x);
    p.logit_s = wsp<float>(c, c->off.logit_s);
    p.err = wsp<unsigned>(c, c->err_off);
    p.n = wsp<int32_t>(c, c->off.n); p.k_eff = wsp<int32_t>(c, c->off.k_eff);
    p.tdepth = tree_depth; p.tanc = reinterpret_cast<const u64*>(tree_anc);   // rows of a candidate tree (null: a chain)
    p.L = c->L; p.d = c->d; p.H = c->H; p.m = c->m; p.Vs = c->Vs; p.S = c->S; p.B = c->B; p.C = c->C;
    p.RS = RS; p.MR = c->S * RS; p.RPJ = RPJ; p.Smax = c->Smax; p.Tmax = c->Tmax;
    p.hd = c->hd; p.qscale = 1.0f / sqrtf((float)c->hd);
    p.KpA = P->KpA; p.KpO = P->KpO; p.KpH = P->KpH;
    p.eps = c->cfg.rms_eps;
    const void* kern = nullptr;
    if (c->d == 1280) {
        // strips per compute wave: QKV 240 / 128 -> 2, Wo 80 / 128 -> 1, W1|W3 432 / 128 -> 4, W2 -> 1, output 1024 / 128 -> 8
        p.lm_rounds = 2;
        kern = RPJ == 1 ? reinterpret_cast<const void*>(verify_xcd_kernel<2, 5, 1, 6, 4, 5, 1, 14, 4, 1>)
                        : reinterpret_cast<const void*>(verify_xcd_kernel<2, 5, 1, 6, 4, 5, 1, 14, 4, 2>);
        if (P->NSW[X_A] > 2 || P->NSW[X_C] > 1 || P->NSW[X_D] > 4 || P->NSW[X_E] > 1 || P->NSW[X_LM] > 8) return -1;
    } else if (c->d == 4096) {
        // streamed: QKV 768 strips / 128 waves -> 6, Wo 256 -> 2, W1|W3 1376 -> 11 (12 with an empty one), W2 256 -> 2 x 3 chunks
        // of its 43 k-tiles, output 512 -> 4
        p.lm_rounds = 1;
        kern = RPJ == 1 ? reinterpret_cast<const void*>(verify_xcd_stream_kernel<6, 2, 12, 2, 43, 4, 1, 128>)
                        : reinterpret_cast<const void*>(verify_xcd_stream_kernel<6, 2, 12, 2, 43, 4, 2, 128>);
        if (P->NSW[X_A] > 6 || P->NSW[X_C] > 2 || P->NSW[X_D] > 12 || P->NSW[X_E] > 2 || P->NSW[X_LM] > 4) return -1;
        for (int x = 0; x < kXcd; ++x)
            if (P->KT[X_A][x] != 16 || P->KT[X_C][x] != 16 || P->KT[X_E][x] != 43) return -1;   // (three parts of the W2 input on both sides)
    } else {
        // d = 768: QKV 144 -> 2, Wo 48 -> 1, W1|W3 256 -> 2, W2 48 -> 1, output 8 in two rounds of 4
        p.lm_rounds = 2;
        kern = RPJ == 1 ? reinterpret_cast<const void*>(verify_xcd_kernel<2, 3, 1, 4, 2, 3, 1, 8, 4, 1>)
                        : reinterpret_cast<const void*>(verify_xcd_kernel<2, 3, 1, 4, 2, 3, 1, 8, 4, 2>);
        if (P->NSW[X_A] > 2 || P->NSW[X_C] > 1 || P->NSW[X_D] > 2 || P->NSW[X_E] > 1 || P->NSW[X_LM] > 8) return -1;
    }
    // the parameter block and the attention job table of this step shape: uploaded when they change
    static_assert(sizeof(XP) <= 4096, "parameter block larger than its workspace region");
    if (P->params.size() != sizeof(XP) || memcmp(P->params.data(), &p, sizeof(XP)) != 0) {
        if (hipMemcpyAsync(c->ws + o.atab, atab.data(), atab.size() * 2, hipMemcpyHostToDevice, c->stream) != hipSuccess) return -1;
        if (hipMemcpyAsync(c->ws + o.xp, &p, sizeof(XP), hipMemcpyHostToDevice, c->stream) != hipSuccess) return -1;
        if (hipStreamSynchronize(c->stream) != hipSuccess) return -1;   // the sources are locals: the copies must have read them
        P->params.assign(reinterpret_cast<const uint8_t*>(&p), reinterpret_cast<const uint8_t*>(&p) + sizeof(XP));
    }
    const size_t lds = xcd_lds_bytes(c, P, RPJ, c->S * RS);
    if (lds > (size_t)160 * 1024) return -1;
    if (hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess) return -1;
    const XP* dev_params = wsp<XP>(c, o.xp);
    unsigned epoch0 = P->epoch;
    u64* dbg = c->stream_dbg ? wsp<u64>(c, o.dbg) : nullptr;
    unsigned par = P->par, par_lm = P->par_lm;
    void* args[] = {&dev_params, &epoch0, &par, &par_lm, &dbg};
    // one workgroup per compute unit: the grid equals the unit count and a workgroup's LDS request
    // (padded to more than half a unit's LDS) keeps a second one off the unit
    const size_t lds_req = std::max(lds, (size_t)84 * 1024);
    if (hipLaunchKernel(kern, dim3(kNWG), dim3(kThreads), args, lds_req, c->stream) != hipSuccess) return -1;
    P->epoch += 5u * (unsigned)(c->L + 2) + 8u;
    // parities of the partial-sum words after this launch: rows in flight were written once per layer into the
    // layer parity's area, once into the output projection's
    const int MR = c->S * RS;
    const unsigned rows = MR >= 16 ? 0xFFFFu : (1u << MR) - 1u;
    if (((c->L + 1) / 2) & 1) P->par ^= rows;
    if ((c->L / 2) & 1) P->par ^= rows << 16;
    P->par_lm ^= rows;
    return 0;
}

}  // namespace hawk
