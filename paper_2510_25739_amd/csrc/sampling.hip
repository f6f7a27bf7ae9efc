// Sampling stage: guidance, temperature / top-k warp, inverse-CDF draws, the accept /
// reject scan with residual resampling, and the commit of a step.
//
// Decisions (which logits survive top-k, where a uniform falls in a CDF, whether a draft is
// accepted) are taken on fp32 logits with fp64 weights exp(z - zmax) and fp64 sums, so
// that they do not depend on the order of summation beyond the last bits of an fp64.
// One workgroup of 1024 threads handles one logit row; thread t owns the contiguous index
// segment [t*E, (t+1)*E), which makes every scan an in-order prefix over token indices.
// Reductions use wavefront shuffles, then one LDS exchange across the 16 waves.
#include <mutex>
#include "hawk_internal.h"

namespace hawk {

namespace {

constexpr int NT = kSampThreads;
constexpr int NW = NT / 64;

struct Shared {
    unsigned hist[256];
    double dred[NW];
    int ired[NW];
    float fred[NW];
    unsigned ukred[NW];
    // broadcast slots
    unsigned b_prefix, b_remaining, b_count_eq;
    int b_int;
    double b_dbl;
};

__device__ __forceinline__ uint64_t mix64(uint64_t z) {
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}
__device__ __forceinline__ float gen_uniform(uint64_t seed, uint32_t seq, uint32_t step, uint32_t slot) {
    uint64_t ctr = ((uint64_t)seq << 44) | ((uint64_t)step << 8) | (uint64_t)(slot & 0xFFu);
    uint64_t z = mix64(seed + 0x9E3779B97F4A7C15ull);
    z = mix64(z + 0x9E3779B97F4A7C15ull * (ctr + 1));
    return (float)(z >> 40) * (1.0f / 16777216.0f);
}
__device__ __forceinline__ float pick_uniform(const UniformSrc& u, const float* table, int idx, int b, int slot) {
    return u.use_gen ? gen_uniform(u.seed, (uint32_t)b, (uint32_t)u.step[0], (uint32_t)slot) : table[idx];
}

// Order-preserving key of a float (larger value <=> larger key); -0 and +0 share a key.
__device__ __forceinline__ unsigned fkey(float z) {
    unsigned u = __float_as_uint(z);
    if ((u << 1) == 0u) u = 0u;
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Cross-lane moves inside the VALU (DPP) instead of LDS-crossbar shuffles: within a row of 16
// lanes by quad permutes and mirrors, across the four rows by lane broadcasts.
template <int CTRL>
__device__ __forceinline__ int dpp_i(int v) { return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xF, 0xF, true); }
template <int CTRL>
__device__ __forceinline__ float dpp_f(float v) { return __builtin_bit_cast(float, dpp_i<CTRL>(__builtin_bit_cast(int, v))); }
template <int CTRL>
__device__ __forceinline__ double dpp_d(double v) {
    const unsigned long long b = __builtin_bit_cast(unsigned long long, v);
    const unsigned lo = (unsigned)dpp_i<CTRL>((int)(unsigned)b), hi = (unsigned)dpp_i<CTRL>((int)(unsigned)(b >> 32));
    return __builtin_bit_cast(double, ((unsigned long long)hi << 32) | lo);
}
__device__ __forceinline__ float lane_f(float v, int l) {
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), l));
}
__device__ __forceinline__ double lane_d(double v, int l) {
    const unsigned long long b = __builtin_bit_cast(unsigned long long, v);
    const unsigned lo = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)b, l);
    const unsigned hi = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)(b >> 32), l);
    return __builtin_bit_cast(double, ((unsigned long long)hi << 32) | lo);
}
// 0xB1 = quad_perm [1,0,3,2], 0x4E = quad_perm [2,3,0,1], 0x141 = row_half_mirror, 0x140 = row_mirror:
// after the four steps every lane of a row holds the row's result.
#define ROW_ALLREDUCE(v, OP, DPP)         \
    v = OP(v, DPP<0xB1>(v));              \
    v = OP(v, DPP<0x4E>(v));              \
    v = OP(v, DPP<0x141>(v));             \
    v = OP(v, DPP<0x140>(v));
__device__ __forceinline__ double addd(double a, double b) { return a + b; }
__device__ __forceinline__ int mini(int a, int b) { return min(a, b); }
__device__ __forceinline__ int maxi(int a, int b) { return max(a, b); }

__device__ __forceinline__ double wave_sum_d(double v) {
    ROW_ALLREDUCE(v, addd, dpp_d)
    return (lane_d(v, 0) + lane_d(v, 16)) + (lane_d(v, 32) + lane_d(v, 48));
}
__device__ __forceinline__ float wave_max_f(float v) {
    ROW_ALLREDUCE(v, fmaxf, dpp_f)
    return fmaxf(fmaxf(lane_f(v, 0), lane_f(v, 16)), fmaxf(lane_f(v, 32), lane_f(v, 48)));
}
__device__ __forceinline__ float wave_min_f(float v) {
    ROW_ALLREDUCE(v, fminf, dpp_f)
    return fminf(fminf(lane_f(v, 0), lane_f(v, 16)), fminf(lane_f(v, 32), lane_f(v, 48)));
}
__device__ __forceinline__ int wave_min_i(int v) {
    ROW_ALLREDUCE(v, mini, dpp_i)
    return min(min(__builtin_amdgcn_readlane(v, 0), __builtin_amdgcn_readlane(v, 16)),
               min(__builtin_amdgcn_readlane(v, 32), __builtin_amdgcn_readlane(v, 48)));
}
__device__ __forceinline__ int wave_max_i(int v) {
    ROW_ALLREDUCE(v, maxi, dpp_i)
    return max(max(__builtin_amdgcn_readlane(v, 0), __builtin_amdgcn_readlane(v, 16)),
               max(__builtin_amdgcn_readlane(v, 32), __builtin_amdgcn_readlane(v, 48)));
}
// Inclusive prefix sums over the lanes of the wave, in lane order: row_shr 1, 2, 4, 8 with zero
// fill inside each row of 16 (0x111, 0x112, 0x114, 0x118), then the totals of the rows before.
__device__ __forceinline__ double wave_incl_scan_d(double v) {
    v += dpp_d<0x111>(v);
    v += dpp_d<0x112>(v);
    v += dpp_d<0x114>(v);
    v += dpp_d<0x118>(v);
    const double r0 = lane_d(v, 15), r1 = lane_d(v, 31), r2 = lane_d(v, 47);
    const int row = (threadIdx.x & 63) >> 4;
    return v + (row == 0 ? 0.0 : row == 1 ? r0 : row == 2 ? r0 + r1 : (r0 + r1) + r2);
}
__device__ __forceinline__ int wave_incl_scan_i(int v) {
    v += dpp_i<0x111>(v);
    v += dpp_i<0x112>(v);
    v += dpp_i<0x114>(v);
    v += dpp_i<0x118>(v);
    const int r0 = __builtin_amdgcn_readlane(v, 15), r1 = __builtin_amdgcn_readlane(v, 31), r2 = __builtin_amdgcn_readlane(v, 47);
    const int row = (threadIdx.x & 63) >> 4;
    return v + (row == 0 ? 0 : row == 1 ? r0 : row == 2 ? r0 + r1 : r0 + r1 + r2);
}

// All block primitives below return the same value to every thread and may be called
// back to back (each starts with a barrier that protects the exchange buffer).
__device__ double block_sum_d(double v, Shared& sh) {
    v = wave_sum_d(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sh.dred[threadIdx.x >> 6] = v;
    __syncthreads();
    double t = 0.0;
#pragma unroll
    for (int w = 0; w < NW; ++w) t += sh.dred[w];
    return t;
}
__device__ float block_max_f(float v, Shared& sh) {
    v = wave_max_f(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sh.fred[threadIdx.x >> 6] = v;
    __syncthreads();
    float t = sh.fred[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) t = fmaxf(t, sh.fred[w]);
    return t;
}
// Minimum and maximum over the block in one exchange.
__device__ void block_minmax_f(float& lo, float& hi, Shared& sh) {
    lo = wave_min_f(lo);
    hi = wave_max_f(hi);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) { sh.fred[threadIdx.x >> 6] = lo; sh.dred[threadIdx.x >> 6] = (double)hi; }
    __syncthreads();
    lo = sh.fred[0]; hi = (float)sh.dred[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) { lo = fminf(lo, sh.fred[w]); hi = fmaxf(hi, (float)sh.dred[w]); }
}
__device__ int block_min_i(int v, Shared& sh) {
    v = wave_min_i(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sh.ired[threadIdx.x >> 6] = v;
    __syncthreads();
    int t = sh.ired[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) t = min(t, sh.ired[w]);
    return t;
}
__device__ int block_max_i(int v, Shared& sh) {
    v = wave_max_i(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sh.ired[threadIdx.x >> 6] = v;
    __syncthreads();
    int t = sh.ired[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) t = max(t, sh.ired[w]);
    return t;
}
// Exclusive prefix sums over the threads of the block, in thread order.
__device__ double block_excl_scan_d(double v, Shared& sh) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const double inc = wave_incl_scan_d(v);
    __syncthreads();
    if (lane == 63) sh.dred[wave] = inc;
    __syncthreads();
    double base = 0.0;
#pragma unroll
    for (int w = 0; w < NW; ++w) base += w < wave ? sh.dred[w] : 0.0;
    return base + (inc - v);
}
__device__ int block_excl_scan_i(int v, Shared& sh) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int inc = wave_incl_scan_i(v);
    __syncthreads();
    if (lane == 63) sh.ired[wave] = inc;
    __syncthreads();
    int base = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) base += w < wave ? sh.ired[w] : 0;
    return base + (inc - v);
}

struct Seg { int j0, j1; };
__device__ __forceinline__ Seg my_segment(int n) {
    int e = (n + NT - 1) / NT;
    Seg s;
    s.j0 = min(n, (int)threadIdx.x * e);
    s.j1 = min(n, s.j0 + e);
    return s;
}

// Guided logits of one row into `out` (also the row every later pass reads).
__device__ void combine_row(const float* lc, const float* lu, float scale, float* out, int n) {
    for (int j = threadIdx.x; j < n; j += NT) out[j] = lu ? fmaf(scale, lc[j] - lu[j], lu[j]) : lc[j];
    __syncthreads();
}

__device__ __forceinline__ bool kept(const WarpStat& st, float z, int j) {
    unsigned k = fkey(z);
    return k > st.tau || (k == st.tau && j <= st.tie_cut);
}
__device__ __forceinline__ double weight_of(const WarpStat& st, const float* l, float inv_t, int j) {
    if (st.onehot >= 0) return j == st.onehot ? 1.0 : 0.0;
    float z = l[j] * inv_t;
    return kept(st, z, j) ? exp((double)z - (double)st.zmax) : 0.0;
}

// Temperature / top-k warp of the row l[0..n): arg-max point mass if greedy, otherwise
// z = l * inv_t, keep the top_k largest z (equal values: lower index first).
__device__ WarpStat warp_stats(const float* l, int n, float inv_t, int top_k, int greedy, Shared& sh) {
    const Seg sg = my_segment(n);
    WarpStat st;
    st.total = 1.0; st.zmax = 0.f; st.tau = 0u; st.tie_cut = 0x7FFFFFFF; st.onehot = -1;
    if (greedy) {
        float best = -INFINITY;
        for (int j = sg.j0; j < sg.j1; ++j) best = fmaxf(best, l[j]);
        float gmax = block_max_f(best, sh);
        int idx = 0x7FFFFFFF;
        for (int j = sg.j0; j < sg.j1; ++j)
            if (l[j] == gmax) { idx = j; break; }
        st.onehot = block_min_i(idx, sh);
        return st;
    }
    const int K = min(top_k, n);
    if (K < n) {
        unsigned prefix = 0u, mask = 0u, remaining = (unsigned)K, count_eq = 0u;
        for (int shift = 24; shift >= 0; shift -= 8) {
            __syncthreads();
            if (threadIdx.x < 256) sh.hist[threadIdx.x] = 0u;
            __syncthreads();
            for (int j = sg.j0; j < sg.j1; ++j) {
                unsigned key = fkey(l[j] * inv_t);
                if ((key & mask) == prefix) atomicAdd(&sh.hist[(key >> shift) & 255u], 1u);
            }
            __syncthreads();
            if (threadIdx.x == 0) {
                unsigned cum = 0u;
                for (int bin = 255; bin >= 0; --bin) {
                    unsigned h = sh.hist[bin];
                    if (cum + h >= remaining) {
                        sh.b_prefix = prefix | ((unsigned)bin << shift);
                        sh.b_remaining = remaining - cum;
                        sh.b_count_eq = h;
                        break;
                    }
                    cum += h;
                }
            }
            __syncthreads();
            prefix = sh.b_prefix;
            remaining = sh.b_remaining;
            count_eq = sh.b_count_eq;
            mask |= 255u << shift;
        }
        st.tau = prefix;
        if (remaining < count_eq) {  // keep only the first `remaining` entries equal to tau
            int c = 0;
            for (int j = sg.j0; j < sg.j1; ++j) c += fkey(l[j] * inv_t) == prefix;
            int before = block_excl_scan_i(c, sh);
            __syncthreads();
            if (before < (int)remaining && before + c >= (int)remaining) {
                int seen = before;
                for (int j = sg.j0; j < sg.j1; ++j)
                    if (fkey(l[j] * inv_t) == prefix && ++seen == (int)remaining) { sh.b_int = j; break; }
            }
            __syncthreads();
            st.tie_cut = sh.b_int;
        }
    }
    float zm = -INFINITY;
    for (int j = sg.j0; j < sg.j1; ++j) zm = fmaxf(zm, l[j] * inv_t);
    st.zmax = block_max_f(zm, sh);
    double s = 0.0;
    for (int j = sg.j0; j < sg.j1; ++j) s += weight_of(st, l, inv_t, j);
    st.total = block_sum_d(s, sh);
    return st;
}

// Inverse-CDF draw over ascending index from weights w(j) >= 0 given by a functor:
// first j whose running sum exceeds u * total, else the last j with positive weight.
template <class WF>
__device__ int inv_cdf(WF w, int n, double total, float u, Shared& sh) {
    const Seg sg = my_segment(n);
    double s = 0.0;
    for (int j = sg.j0; j < sg.j1; ++j) s += w(j);
    double c = block_excl_scan_d(s, sh);
    const double target = (double)u * total;
    int cand = 0x7FFFFFFF, last = -1;
    for (int j = sg.j0; j < sg.j1; ++j) {
        double wj = w(j);
        if (wj > 0.0) {
            c += wj;
            last = j;
            if (c > target) { cand = j; break; }
        }
    }
    cand = block_min_i(cand, sh);
    if (cand != 0x7FFFFFFF) return cand;
    return block_max_i(last, sh);
}

// ---------------------------------------------------------------------------- kernels

__global__ void plan_kernel(const int32_t* n, int32_t* k_eff, int32_t* draft, int32_t* step,
                            unsigned long long* counters, int B, int N, int k, int kstride) {
    int b = threadIdx.x;
    if (b == 0) {
        step[0] += 1;
        bool any = false;
        for (int j = 0; j < B; ++j) any = any || n[j] < N;
        if (any) counters[3] += 1ull;  // lock-step iterations that still had work
    }
    if (b >= B) return;
    int nb = n[b];
    k_eff[b] = nb < N ? min(k, N - nb - 1) : -1;
    for (int i = 0; i < kstride; ++i) draft[b * kstride + i] = -1;
}

struct SampParams {
    int B, N, Vs, samp_lo, kstride, top_k, greedy, use_cfg;
    float inv_t, cfg_scale;
};

// Token 0 of every prompt from the logits of the last condition row.
__global__ __launch_bounds__(NT) void first_token_kernel(const float* logit_s, float* logit_b, int32_t* grid,
                                                         int32_t* n, SampParams P, UniformSrc us) {
    __shared__ Shared sh;
    const int b = blockIdx.x;
    float* row = logit_b + (size_t)b * P.kstride * P.Vs;
    combine_row(logit_s + (size_t)b * P.Vs, P.use_cfg ? logit_s + (size_t)(P.B + b) * P.Vs : nullptr,
                P.cfg_scale, row, P.Vs);
    WarpStat st = warp_stats(row, P.Vs, P.inv_t, P.top_k, P.greedy, sh);
    float u = pick_uniform(us, us.fin, b, b, kSlotFinal);
    int idx = inv_cdf([&](int j) { return weight_of(st, row, P.inv_t, j); }, P.Vs, st.total, u, sh);
    if (threadIdx.x == 0) {
        grid[(size_t)b * P.N] = P.samp_lo + idx;
        n[b] = 1;
    }
}

// Draft i (1-based): guide, warp, then draw the token by inverse CDF - or, when a table
// of forced tokens is given, take the token from it (teacher-forced drafting; with
// point_mass the draft distribution becomes the point mass on that token).  Keeps the
// guided row and its warp statistics for the accept test of the verify step.
struct ForcedSrc {
    const int32_t* table;  // nullptr: sample
    int32_t stride;        // row stride of the table
    int32_t relative;      // 1: column n[b] + i - 1 (replay grid), 0: column i - 1
    int32_t point_mass;
};

__global__ __launch_bounds__(NT) void draft_sample_kernel(const float* dlogit_s, float* dlogit_b, const int32_t* n,
                                                          const int32_t* k_eff, int32_t* draft, WarpStat* qstat,
                                                          int i, int k, SampParams P, UniformSrc us, ForcedSrc fs) {
    __shared__ Shared sh;
    const int b = blockIdx.x;
    if (i > k_eff[b]) return;
    float* row = dlogit_b + ((size_t)b * P.kstride + (i - 1)) * P.Vs;
    combine_row(dlogit_s + (size_t)b * P.Vs, P.use_cfg ? dlogit_s + (size_t)(P.B + b) * P.Vs : nullptr,
                P.cfg_scale, row, P.Vs);
    WarpStat st = warp_stats(row, P.Vs, P.inv_t, P.top_k, P.greedy, sh);
    int tok;
    if (fs.table) {
        tok = fs.table[(size_t)b * fs.stride + (fs.relative ? n[b] : 0) + (i - 1)];
        if (fs.point_mass) { st.onehot = tok - P.samp_lo; st.total = 1.0; }
    } else {
        float u = pick_uniform(us, us.draft, b * k + (i - 1), b, kSlotDraft + (i - 1));
        tok = P.samp_lo + inv_cdf([&](int j) { return weight_of(st, row, P.inv_t, j); }, P.Vs, st.total, u, sh);
    }
    if (threadIdx.x == 0) {
        draft[b * P.kstride + (i - 1)] = tok;
        qstat[b * P.kstride + (i - 1)] = st;
    }
}

// Guided target row r of prompt b and its warp statistics.
__global__ __launch_bounds__(NT) void verify_stats_kernel(const float* logit_s, float* logit_b,
                                                          const int32_t* k_eff, WarpStat* pstat, int k,
                                                          SampParams P) {
    __shared__ Shared sh;
    const int r = blockIdx.x, b = blockIdx.y;
    if (r > k_eff[b]) return;
    float* row = logit_b + ((size_t)b * P.kstride + r) * P.Vs;
    combine_row(logit_s + ((size_t)b * (k + 1) + r) * P.Vs,
                P.use_cfg ? logit_s + ((size_t)(P.B + b) * (k + 1) + r) * P.Vs : nullptr, P.cfg_scale, row, P.Vs);
    WarpStat st = warp_stats(row, P.Vs, P.inv_t, P.top_k, P.greedy, sh);
    if (threadIdx.x == 0) pstat[b * P.kstride + r] = st;
}

// Accept scan, residual / bonus draw and commit for prompt b.
__global__ __launch_bounds__(NT) void accept_commit_kernel(
    const float* logit_b, const float* dlogit_b, const WarpStat* pstat, const WarpStat* qstat, const int32_t* k_eff,
    const int32_t* draft, int32_t* grid, int32_t* n, const uint32_t* hid, uint32_t* hprev, int hid_words,
    int32_t* out_na, int32_t* out_tok, unsigned long long* counters, int k, int n_seq_streams, SampParams P,
    UniformSrc us) {
    __shared__ Shared sh;
    const int b = blockIdx.x;
    const int ke = k_eff[b];
    if (threadIdx.x <= k) out_tok[b * (k + 1) + threadIdx.x] = -1;
    if (ke < 0) {
        if (threadIdx.x == 0) out_na[b] = -1;
        return;
    }
    // accept scan (every thread computes the same thing)
    int a = 0;
    for (; a < ke; ++a) {
        const int dj = draft[b * P.kstride + a] - P.samp_lo;
        const WarpStat ps = pstat[b * P.kstride + a], qs = qstat[b * P.kstride + a];
        const double pd = weight_of(ps, logit_b + ((size_t)b * P.kstride + a) * P.Vs, P.inv_t, dj) / ps.total;
        const double qd = weight_of(qs, dlogit_b + ((size_t)b * P.kstride + a) * P.Vs, P.inv_t, dj) / qs.total;
        const float u = pick_uniform(us, us.acc, b * k + a, b, kSlotAcc + a);
        if (!((double)u * qd < pd)) break;
    }
    const float uf = pick_uniform(us, us.fin, b, b, kSlotFinal);
    const float* prow = logit_b + ((size_t)b * P.kstride + a) * P.Vs;
    const WarpStat ps = pstat[b * P.kstride + a];
    int y;
    auto wp = [&](int j) { return weight_of(ps, prow, P.inv_t, j); };
    if (a < ke) {
        const float* qrow = dlogit_b + ((size_t)b * P.kstride + a) * P.Vs;
        const WarpStat qs = qstat[b * P.kstride + a];
        auto res = [&](int j) {
            double r = weight_of(ps, prow, P.inv_t, j) / ps.total - weight_of(qs, qrow, P.inv_t, j) / qs.total;
            return r > 0.0 ? r : 0.0;
        };
        const Seg sg = my_segment(P.Vs);
        double s = 0.0;
        for (int j = sg.j0; j < sg.j1; ++j) s += res(j);
        const double R = block_sum_d(s, sh);
        y = (R > 0.0) ? inv_cdf(res, P.Vs, R, uf, sh) : inv_cdf(wp, P.Vs, ps.total, uf, sh);
    } else {
        y = inv_cdf(wp, P.Vs, ps.total, uf, sh);
    }
    // commit: tokens, counters, hidden state of row a for the next draft
    const int nb = n[b];
    for (int s = b; s < n_seq_streams; s += P.B) {
        const uint32_t* src = hid + ((size_t)s * (k + 1) + a) * hid_words;
        uint32_t* dst = hprev + (size_t)s * hid_words;
        for (int i = threadIdx.x; i < hid_words; i += NT) dst[i] = src[i];
    }
    __syncthreads();  // every thread has read n[b] before it changes
    if (threadIdx.x == 0) {
        for (int i = 0; i < a; ++i) {
            int t = draft[b * P.kstride + i];
            grid[(size_t)b * P.N + nb + i] = t;
            out_tok[b * (k + 1) + i] = t;
        }
        grid[(size_t)b * P.N + nb + a] = P.samp_lo + y;
        out_tok[b * (k + 1) + a] = P.samp_lo + y;
        out_na[b] = a;
        n[b] = nb + a + 1;
        atomicAdd(&counters[0], 1ull);
        atomicAdd(&counters[1], (unsigned long long)a);
        atomicAdd(&counters[2], (unsigned long long)(a + 1));
    }
}

__global__ void force_setup_kernel(const int32_t* n_from, const int32_t* forced, int32_t* n, int32_t* k_eff,
                                   int32_t* draft, int B, int cnt, int kstride) {
    int b = threadIdx.x;
    if (b >= B) return;
    n[b] = n_from[b];
    k_eff[b] = cnt - 1;
    for (int i = 0; i < kstride; ++i) draft[b * kstride + i] = i < cnt - 1 ? forced[b * cnt + i] : -1;
}

__global__ void force_commit_kernel(const int32_t* forced, int32_t* grid, int32_t* n, const uint32_t* hid,
                                    uint32_t* hprev, int hid_words, int B, int N, int cnt, int n_seq_streams) {
    const int b = blockIdx.x;
    const int nb = n[b];
    for (int s = b; s < n_seq_streams; s += B) {
        const uint32_t* src = hid + ((size_t)s * cnt + (cnt - 1)) * hid_words;
        uint32_t* dst = hprev + (size_t)s * hid_words;
        for (int i = threadIdx.x; i < hid_words; i += blockDim.x) dst[i] = src[i];
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int i = 0; i < cnt; ++i) grid[(size_t)b * N + nb + i] = forced[b * cnt + i];
        n[b] = nb + cnt;
    }
}

// ---------------------------------------------------------------------------- register-resident rows
//
// Fast variants for rows of at most 1024 * E entries: a thread keeps its E scaled logits in
// registers for the whole kernel (one coalesced read of the row), the radix select counts
// digits in per-wave LDS histograms (all logits of a row share their high bits, so a single
// shared histogram serialises on two or three counters), the digit scan runs on one wave, and
// the fp64 weights exp(z - zmax) are computed once and reused by the sum and by the
// inverse-CDF scan.  Same decisions, to the bit, as the generic functions above.

constexpr int kCand = 256;   // entries of the threshold's first-digit bin that are ranked directly
struct FastShared {
    unsigned hist[NW][256];
    unsigned tot[256];
    alignas(16) unsigned cand_rel[kCand];
    int cand_idx[kCand];
    unsigned cand_rank[kCand];   // candidates that come before each one (see rank_candidates)
    unsigned cand_n;
    Shared sh;
};

// Ranks of all gathered candidates at once (fs.cand_rank[i] = candidates that come before candidate
// i - larger key first, lower index first among equal keys -, zeroed by the caller): the cnt x cnt comparisons are spread over the block - NT / cnt threads share a
// candidate, each compares it with a slice of the list and adds its count with one LDS atomic -
// instead of one wave walking the whole list per 64 candidates.  All threads call; ends with a barrier.
__device__ __forceinline__ void rank_candidates(FastShared& fs, unsigned cnt) {
    const unsigned per = max(1u, (unsigned)NT / cnt), len = (cnt + per - 1u) / per;
    const unsigned i = threadIdx.x % cnt, c = threadIdx.x / cnt;
    if (c < per) {
        const unsigned mine = fs.cand_rel[i];
        const int mi = fs.cand_idx[i];
        const unsigned j1 = min(cnt, (c + 1u) * len);
        unsigned part = 0u;
        for (unsigned j = c * len; j < j1; ++j) {
            const unsigned r = fs.cand_rel[j];
            part += (r > mine || (r == mine && fs.cand_idx[j] < mi)) ? 1u : 0u;
        }
        if (part) atomicAdd(&fs.cand_rank[i], part);
    }
    __syncthreads();
}

// Inverse of fkey (the key of -0 maps back to +0).
__device__ __forceinline__ float key_to_float(unsigned k) {
    return __uint_as_float((k & 0x80000000u) ? (k ^ 0x80000000u) : ~k);
}

template <int E>
__device__ __forceinline__ void load_row(const float* lc, const float* lu, float scale, float inv_t, float* out, int n,
                                         float (&z)[E]) {
    const int base = threadIdx.x * E;
    if ((n & 3) == 0 && (E & 3) == 0 && base + E <= n) {
#pragma unroll
        for (int q = 0; q < E / 4; ++q) {
            float4 a = *reinterpret_cast<const float4*>(lc + base + 4 * q);
            if (lu) {
                const float4 u = *reinterpret_cast<const float4*>(lu + base + 4 * q);
                a.x = fmaf(scale, a.x - u.x, u.x); a.y = fmaf(scale, a.y - u.y, u.y);
                a.z = fmaf(scale, a.z - u.z, u.z); a.w = fmaf(scale, a.w - u.w, u.w);
            }
            if (out) *reinterpret_cast<float4*>(out + base + 4 * q) = a;
            z[4 * q] = a.x * inv_t; z[4 * q + 1] = a.y * inv_t; z[4 * q + 2] = a.z * inv_t; z[4 * q + 3] = a.w * inv_t;
        }
    } else {
#pragma unroll
        for (int e = 0; e < E; ++e) {
            const int j = base + e;
            if (j < n) {
                const float l = lu ? fmaf(scale, lc[j] - lu[j], lu[j]) : lc[j];
                if (out) out[j] = l;
                z[e] = l * inv_t;
            } else {
                z[e] = -INFINITY;  // its key lies below that of every finite value
            }
        }
    }
}

// Which entries of the row held in z the warp keeps (see warp_stats): arg-max, top-k threshold
// and tie cut, maximum.  The weights themselves come from dense_weights or from a CompactList.
// *kmask: bit e set iff the thread's entry e is kept (not set in the greedy case).
template <int E>
__device__ __forceinline__ WarpStat warp_select(const float (&z)[E], int n, int top_k, int greedy, FastShared& fs, unsigned* kmask) {
    Shared& sh = fs.sh;
    const int base = threadIdx.x * E, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    WarpStat st;
    st.total = 1.0; st.zmax = 0.f; st.tau = 0x007FFFFFu; st.tie_cut = -1; st.onehot = -1;  // keeps every finite entry
    *kmask = 0u;
    if (greedy) {
        float best = -INFINITY;
#pragma unroll
        for (int e = 0; e < E; ++e) best = fmaxf(best, z[e]);
        const float gmax = block_max_f(best, sh);
        int idx = 0x7FFFFFFF;
#pragma unroll
        for (int e = E - 1; e >= 0; --e)
            if (base + e < n && z[e] == gmax) idx = base + e;
        st.onehot = block_min_i(idx, sh);
        return st;
    }
    const int K = min(top_k, n);
    if (K < n) {
        // The keys of a row share their high bits (sign, most of the exponent): radix digits are
        // taken from (key - smallest key) shifted up to the top bit, so that the first digit
        // already spreads the row over the 256 bins (few LDS atomics collide, fewer passes).
        float gmin = INFINITY, gmax = -INFINITY;
#pragma unroll
        for (int e = 0; e < E; ++e)
            if (base + e < n) { gmin = fminf(gmin, z[e]); gmax = fmaxf(gmax, z[e]); }
        block_minmax_f(gmin, gmax, sh);
        const unsigned kmin = fkey(gmin), kmax = fkey(gmax);  // the key order is the value order
        const int sh0 = kmax > kmin ? __clz((int)(kmax - kmin)) : 31;
        // First the row is cut into 256 bins that are linear in the value (the float keys are
        // logarithmic: two or three of their first digits would hold nearly everything); the
        // threshold's bin then holds a few dozen entries, which are ranked directly.  If it holds
        // too many (ties, odd distributions), the exact radix select on the keys takes over.
        bool lin = gmax > gmin && gmin > -INFINITY && gmax < INFINITY;
        const float scale = lin ? 255.99f / (gmax - gmin) : 0.f;
        unsigned rel[E];
#pragma unroll
        for (int e = 0; e < E; ++e) rel[e] = (fkey(z[e]) - kmin) << sh0;
        unsigned prefix = 0u, mask = 0u, remaining = (unsigned)K, count_eq = 0u;
        int ranked_cut = -1;
        for (int shift = 24; shift >= 0 && shift + 8 > sh0;) {  // digits below bit sh0 are all zero
            __syncthreads();
#pragma unroll
            for (int q = 0; q < 4; ++q) fs.hist[wave][lane * 4 + q] = 0u;
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int e = 0; e < E; ++e) {
                const unsigned digit = lin ? min(255u, (unsigned)((z[e] - gmin) * scale)) : ((rel[e] >> shift) & 255u);
                if (base + e < n && (lin || (rel[e] & mask) == prefix)) atomicAdd(&fs.hist[wave][digit], 1u);
            }
            __syncthreads();
            if (threadIdx.x < 256) {
                unsigned t = 0u;
#pragma unroll
                for (int q = 0; q < NW; ++q) t += fs.hist[q][threadIdx.x];
                fs.tot[threadIdx.x] = t;
            }
            __syncthreads();
            if (wave == 0) {  // lane owns bins 4*lane .. 4*lane+3; suffix sums from the top bin down
                const unsigned c0 = fs.tot[lane * 4], c1 = fs.tot[lane * 4 + 1], c2 = fs.tot[lane * 4 + 2], c3 = fs.tot[lane * 4 + 3];
                unsigned suf = c0 + c1 + c2 + c3;  // inclusive suffix over lanes >= this one
#pragma unroll
                for (int o = 1; o < 64; o <<= 1) {
                    const unsigned t = __shfl_down(suf, o, 64);
                    if (lane + o < 64) suf += t;
                }
                const unsigned above = suf - (c0 + c1 + c2 + c3);  // entries in higher lanes' bins
                // highest bin b with (entries in bins >= b) >= remaining
                int found = -1;
                unsigned rem_out = 0u, cnt_out = 0u;
                unsigned cum = above;
                const unsigned cs[4] = {c0, c1, c2, c3};
#pragma unroll
                for (int q = 3; q >= 0; --q) {
                    if (found < 0 && cum < remaining && cum + cs[q] >= remaining) {
                        found = lane * 4 + q; rem_out = remaining - cum; cnt_out = cs[q];
                    }
                    cum += cs[q];
                }
                if (found >= 0) {  // exactly one lane finds it
                    sh.b_prefix = lin ? (unsigned)found : (prefix | ((unsigned)found << shift));
                    sh.b_remaining = rem_out;
                    sh.b_count_eq = cnt_out;
                }
            }
            __syncthreads();
            if (lin) {
                const unsigned bin = sh.b_prefix, want = sh.b_remaining, cnt = sh.b_count_eq;
                if (cnt > (unsigned)kCand) { lin = false; continue; }  // same digit again, on the keys
                if (threadIdx.x == 0) fs.cand_n = 0u;
                if (threadIdx.x < (unsigned)kCand) fs.cand_rank[threadIdx.x] = 0u;
                __syncthreads();
#pragma unroll
                for (int e = 0; e < E; ++e)
                    if (base + e < n && min(255u, (unsigned)((z[e] - gmin) * scale)) == bin) {
                        const unsigned at = atomicAdd(&fs.cand_n, 1u);
                        if (at < (unsigned)kCand) { fs.cand_rel[at] = rel[e]; fs.cand_idx[at] = base + e; }
                    }
                __syncthreads();
                rank_candidates(fs, cnt);
                if (threadIdx.x < cnt && fs.cand_rank[threadIdx.x] + 1u == want) { sh.b_prefix = fs.cand_rel[threadIdx.x]; sh.b_int = fs.cand_idx[threadIdx.x]; }
                __syncthreads();
                prefix = sh.b_prefix;
                ranked_cut = sh.b_int;
                break;
            }
            prefix = sh.b_prefix;
            remaining = sh.b_remaining;
            count_eq = sh.b_count_eq;
            mask |= 255u << shift;
            if (shift == 24 && count_eq <= (unsigned)kCand) {
                // Few entries share the threshold's first digit: gather them and rank each one
                // directly (larger value first, lower index first among equals); the entry of
                // rank `remaining` is the threshold and the tie cut in one.
                if (threadIdx.x == 0) fs.cand_n = 0u;
                if (threadIdx.x < (unsigned)kCand) fs.cand_rank[threadIdx.x] = 0u;
                __syncthreads();
#pragma unroll
                for (int e = 0; e < E; ++e)
                    if (base + e < n && (rel[e] & mask) == prefix) {
                        const unsigned at = atomicAdd(&fs.cand_n, 1u);
                        if (at < (unsigned)kCand) { fs.cand_rel[at] = rel[e]; fs.cand_idx[at] = base + e; }
                    }
                __syncthreads();
                rank_candidates(fs, count_eq);
                if (threadIdx.x < count_eq && fs.cand_rank[threadIdx.x] + 1u == remaining) { sh.b_prefix = fs.cand_rel[threadIdx.x]; sh.b_int = fs.cand_idx[threadIdx.x]; }
                __syncthreads();
                prefix = sh.b_prefix;
                ranked_cut = sh.b_int;
                break;
            }
            if (count_eq == 1u && shift > 0) {  // a single entry is left under the prefix: it is the K-th
                __syncthreads();
#pragma unroll
                for (int e = 0; e < E; ++e)
                    if (base + e < n && (rel[e] & mask) == prefix) sh.b_prefix = rel[e];
                __syncthreads();
                prefix = sh.b_prefix;
                break;
            }
            shift -= 8;
        }
        st.tau = (prefix >> sh0) + kmin;
        st.tie_cut = 0x7FFFFFFF;
        if (ranked_cut >= 0) {
            st.tie_cut = ranked_cut;
        } else if (remaining < count_eq) {  // keep only the first `remaining` entries equal to tau
            int c = 0;
#pragma unroll
            for (int e = 0; e < E; ++e) c += (base + e < n && rel[e] == prefix) ? 1 : 0;
            const int before = block_excl_scan_i(c, sh);
            __syncthreads();
            if (before < (int)remaining && before + c >= (int)remaining) {
                int seen = before;
#pragma unroll
                for (int e = 0; e < E; ++e)
                    if (base + e < n && rel[e] == prefix && ++seen == (int)remaining) sh.b_int = base + e;
            }
            __syncthreads();
            st.tie_cut = sh.b_int;
        }
        unsigned km = 0u;
#pragma unroll
        for (int e = 0; e < E; ++e)
            km |= (base + e < n && (rel[e] > prefix || (rel[e] == prefix && base + e <= st.tie_cut))) ? (1u << e) : 0u;
        *kmask = km;
        st.zmax = gmax;  // the largest entry is always kept
        return st;
    }
    float zm = -INFINITY;
#pragma unroll
    for (int e = 0; e < E; ++e) zm = fmaxf(zm, z[e]);
    st.zmax = block_max_f(zm, sh);
#pragma unroll
    for (int e = 0; e < E; ++e) *kmask |= (base + e < n && kept(st, z[e], base + e)) ? (1u << e) : 0u;
    return st;
}

template <int E>
__device__ __forceinline__ unsigned kept_mask(const WarpStat& st, const float (&z)[E], int n) {
    const int base = threadIdx.x * E;
    unsigned km = 0u;
#pragma unroll
    for (int e = 0; e < E; ++e) km |= (base + e < n && kept(st, z[e], base + e)) ? (1u << e) : 0u;
    return km;
}

// Weight of every entry of the row in registers; sets st.total.
template <int E>
__device__ void dense_weights(WarpStat& st, const float (&z)[E], double (&w)[E], Shared& sh) {
    const int base = threadIdx.x * E;
    if (st.onehot >= 0) {
#pragma unroll
        for (int e = 0; e < E; ++e) w[e] = (base + e == st.onehot) ? 1.0 : 0.0;
        st.total = 1.0;
        return;
    }
    double s = 0.0;
#pragma unroll
    for (int e = 0; e < E; ++e) {
        w[e] = kept(st, z[e], base + e) ? exp((double)z[e] - (double)st.zmax) : 0.0;
        s += w[e];
    }
    st.total = block_sum_d(s, sh);
}

// When top-k keeps at most kCap entries, they are gathered - in index order - into a list in
// LDS and the fp64 exponentials are evaluated for those only (the other 15 of 16 entries of a
// 16384-entry row would cost a software exp each for a weight of zero).
constexpr int kCap = 2048;
struct CompactList {
    int idx[kCap];
    float z[kCap];
    double w[kCap];
};

__host__ __device__ __forceinline__ bool use_list(int top_k, int n, int greedy) { return !greedy && top_k < n && top_k <= kCap; }

template <int E>
__device__ int compact_row(unsigned kmask, const float (&z)[E], CompactList& L, Shared& sh) {
    const int base = threadIdx.x * E;
    const int c = __popc(kmask);
    int at = block_excl_scan_i(c, sh);
    if (threadIdx.x == NT - 1) sh.b_int = at + c;
#pragma unroll
    for (int e = 0; e < E; ++e)
        if ((kmask >> e) & 1u) {
            if (at < kCap) { L.idx[at] = base + e; L.z[at] = z[e]; }
            ++at;
        }
    __syncthreads();
    return min(sh.b_int, kCap);
}

// w[i] = exp(z[i] - zmax) over the list (thread t owns entries 2t, 2t+1); returns the sum.
__device__ double list_weights(CompactList& L, int Kc, float zmax, Shared& sh) {
    const int i0 = threadIdx.x * 2;
    double s = 0.0;
#pragma unroll
    for (int q = 0; q < 2; ++q)
        if (i0 + q < Kc) {
            const double w = exp((double)L.z[i0 + q] - (double)zmax);
            L.w[i0 + q] = w;
            s += w;
        }
    return block_sum_d(s, sh);
}

// Inverse-CDF draw over list weights w (ascending index order); returns the token index.
__device__ int list_inv_cdf(const double* w, const int* idx, int Kc, double total, float u, Shared& sh) {
    const int i0 = threadIdx.x * 2;
    __syncthreads();  // the weights were written by other threads
    const double w0 = i0 < Kc ? w[i0] : 0.0, w1 = i0 + 1 < Kc ? w[i0 + 1] : 0.0;
    double c = block_excl_scan_d(w0 + w1, sh);
    const double target = (double)u * total;
    int cand = 0x7FFFFFFF, last = -1;
    if (w0 > 0.0) { c += w0; last = i0; if (c > target) cand = i0; }
    if (w1 > 0.0) { c += w1; last = i0 + 1; if (c > target && cand == 0x7FFFFFFF) cand = i0 + 1; }
    cand = block_min_i(cand, sh);
    if (cand != 0x7FFFFFFF) return idx[cand];
    last = block_max_i(last, sh);
    return idx[max(last, 0)];
}

template <int E>
__device__ int inv_cdf_row(const double (&w)[E], double total, float u, Shared& sh);

// One row, start to finish: the warp's statistics (with total) and, if u != null, a draw.
template <int E>
__device__ WarpStat warp_and_draw(const float (&z)[E], int n, int top_k, int greedy, FastShared& fs, CompactList& L,
                                  const float* u, int* drawn) {
    unsigned kmask = 0u;
    WarpStat st = warp_select<E>(z, n, top_k, greedy, fs, &kmask);
    if (st.onehot >= 0) {
        st.total = 1.0;
        if (u) *drawn = st.onehot;
    } else if (use_list(top_k, n, greedy)) {
        const int Kc = compact_row<E>(kmask, z, L, fs.sh);
        st.total = list_weights(L, Kc, st.zmax, fs.sh);
        if (u) *drawn = list_inv_cdf(L.w, L.idx, Kc, st.total, *u, fs.sh);
    } else {
        double w[E];
        dense_weights<E>(st, z, w, fs.sh);
        if (u) *drawn = inv_cdf_row<E>(w, st.total, *u, fs.sh);
    }
    return st;
}

// Inverse-CDF draw from the per-thread weights w (ascending index order).
template <int E>
__device__ int inv_cdf_row(const double (&w)[E], double total, float u, Shared& sh) {
    const int base = threadIdx.x * E;
    double s = 0.0;
#pragma unroll
    for (int e = 0; e < E; ++e) s += w[e];
    double c = block_excl_scan_d(s, sh);
    const double target = (double)u * total;
    int cand = 0x7FFFFFFF, last = -1;
#pragma unroll
    for (int e = 0; e < E; ++e) {
        if (w[e] > 0.0) {
            c += w[e];
            last = base + e;
            if (c > target && cand == 0x7FFFFFFF) cand = base + e;
        }
    }
    cand = block_min_i(cand, sh);
    if (cand != 0x7FFFFFFF) return cand;
    return block_max_i(last, sh);
}

template <int E>
__global__ __launch_bounds__(NT) void first_token_fast(const float* logit_s, float* logit_b, int32_t* grid, int32_t* n,
                                                       SampParams P, UniformSrc us) {
    __shared__ FastShared fs;
    __shared__ CompactList L;
    const int b = blockIdx.x;
    float z[E];
    load_row<E>(logit_s + (size_t)b * P.Vs, P.use_cfg ? logit_s + (size_t)(P.B + b) * P.Vs : nullptr, P.cfg_scale,
                P.inv_t, logit_b + (size_t)b * P.kstride * P.Vs, P.Vs, z);
    const float u = pick_uniform(us, us.fin, b, b, kSlotFinal);
    int idx = 0;
    (void)warp_and_draw<E>(z, P.Vs, P.top_k, P.greedy, fs, L, &u, &idx);
    if (threadIdx.x == 0) {
        grid[(size_t)b * P.N] = P.samp_lo + idx;
        n[b] = 1;
    }
}

template <int E>
__global__ __launch_bounds__(NT) void draft_sample_fast(const float* dlogit_s, float* dlogit_b, const int32_t* n,
                                                        const int32_t* k_eff, int32_t* draft, WarpStat* qstat, int i,
                                                        int k, SampParams P, UniformSrc us, ForcedSrc fsrc) {
    __shared__ FastShared fs;
    __shared__ CompactList L;
    const int b = blockIdx.x;
    if (i > k_eff[b]) return;
    float z[E];
    load_row<E>(dlogit_s + (size_t)b * P.Vs, P.use_cfg ? dlogit_s + (size_t)(P.B + b) * P.Vs : nullptr, P.cfg_scale,
                P.inv_t, dlogit_b + ((size_t)b * P.kstride + (i - 1)) * P.Vs, P.Vs, z);
    const float u = fsrc.table ? 0.f : pick_uniform(us, us.draft, b * k + (i - 1), b, kSlotDraft + (i - 1));
    int drawn = 0;
    WarpStat st = warp_and_draw<E>(z, P.Vs, P.top_k, P.greedy, fs, L, fsrc.table ? nullptr : &u, &drawn);
    int tok;
    if (fsrc.table) {
        tok = fsrc.table[(size_t)b * fsrc.stride + (fsrc.relative ? n[b] : 0) + (i - 1)];
        if (fsrc.point_mass) { st.onehot = tok - P.samp_lo; st.total = 1.0; }
    } else {
        tok = P.samp_lo + drawn;
    }
    if (threadIdx.x == 0) {
        draft[b * P.kstride + (i - 1)] = tok;
        qstat[b * P.kstride + (i - 1)] = st;
    }
}

template <int E>
__global__ __launch_bounds__(NT) void verify_stats_fast(const float* logit_s, float* logit_b, const int32_t* k_eff,
                                                        WarpStat* pstat, int k, SampParams P) {
    __shared__ FastShared fs;
    __shared__ CompactList L;
    const int r = blockIdx.x, b = blockIdx.y;
    if (r > k_eff[b]) return;
    float z[E];
    load_row<E>(logit_s + ((size_t)b * (k + 1) + r) * P.Vs,
                P.use_cfg ? logit_s + ((size_t)(P.B + b) * (k + 1) + r) * P.Vs : nullptr, P.cfg_scale, P.inv_t,
                logit_b + ((size_t)b * P.kstride + r) * P.Vs, P.Vs, z);
    const WarpStat st = warp_and_draw<E>(z, P.Vs, P.top_k, P.greedy, fs, L, nullptr, nullptr);
    if (threadIdx.x == 0) pstat[b * P.kstride + r] = st;
}

template <int E>
__global__ __launch_bounds__(NT) void accept_commit_fast(
    const float* logit_b, const float* dlogit_b, const WarpStat* pstat, const WarpStat* qstat, const int32_t* k_eff,
    const int32_t* draft, int32_t* grid, int32_t* n, const uint32_t* hid, uint32_t* hprev, int hid_words,
    int32_t* out_na, int32_t* out_tok, unsigned long long* counters, int k, int n_seq_streams, SampParams P,
    UniformSrc us) {
    __shared__ Shared sh;
    __shared__ CompactList L;
    __shared__ double res_list[kCap];
    const int b = blockIdx.x;
    const int ke = k_eff[b];
    if (threadIdx.x <= k) out_tok[b * (k + 1) + threadIdx.x] = -1;
    if (ke < 0) {
        if (threadIdx.x == 0) out_na[b] = -1;
        return;
    }
    int a = 0;
    for (; a < ke; ++a) {
        const int dj = draft[b * P.kstride + a] - P.samp_lo;
        const WarpStat ps = pstat[b * P.kstride + a], qs = qstat[b * P.kstride + a];
        const double pd = weight_of(ps, logit_b + ((size_t)b * P.kstride + a) * P.Vs, P.inv_t, dj) / ps.total;
        const double qd = weight_of(qs, dlogit_b + ((size_t)b * P.kstride + a) * P.Vs, P.inv_t, dj) / qs.total;
        const float u = pick_uniform(us, us.acc, b * k + a, b, kSlotAcc + a);
        if (!((double)u * qd < pd)) break;
    }
    const float uf = pick_uniform(us, us.fin, b, b, kSlotFinal);
    const float* prow = logit_b + ((size_t)b * P.kstride + a) * P.Vs;
    const WarpStat ps = pstat[b * P.kstride + a];
    const int base = threadIdx.x * E;
    int y;
    if (ps.onehot < 0 && use_list(P.top_k, P.Vs, P.greedy)) {
        // the kept entries of p (a superset of the residual's support) as a list; q only where p > 0
        float z[E];
        load_row<E>(prow, nullptr, 0.f, P.inv_t, nullptr, P.Vs, z);
        const int Kc = compact_row<E>(kept_mask<E>(ps, z, P.Vs), z, L, sh);
        (void)list_weights(L, Kc, ps.zmax, sh);
        if (a < ke) {
            const float* qrow = dlogit_b + ((size_t)b * P.kstride + a) * P.Vs;
            const WarpStat qs = qstat[b * P.kstride + a];
            const int i0 = threadIdx.x * 2;
            double s = 0.0;
#pragma unroll
            for (int q2 = 0; q2 < 2; ++q2)
                if (i0 + q2 < Kc) {
                    const double q = weight_of(qs, qrow, P.inv_t, L.idx[i0 + q2]) / qs.total;
                    const double r = L.w[i0 + q2] / ps.total - q;
                    res_list[i0 + q2] = r > 0.0 ? r : 0.0;
                    s += res_list[i0 + q2];
                }
            const double R = block_sum_d(s, sh);
            y = (R > 0.0) ? list_inv_cdf(res_list, L.idx, Kc, R, uf, sh) : list_inv_cdf(L.w, L.idx, Kc, ps.total, uf, sh);
        } else {
            y = list_inv_cdf(L.w, L.idx, Kc, ps.total, uf, sh);
        }
    } else {
    double w[E];
#pragma unroll
    for (int e = 0; e < E; ++e) w[e] = base + e < P.Vs ? weight_of(ps, prow, P.inv_t, base + e) : 0.0;
    if (a < ke) {
        const float* qrow = dlogit_b + ((size_t)b * P.kstride + a) * P.Vs;
        const WarpStat qs = qstat[b * P.kstride + a];
        double res[E], s = 0.0;
#pragma unroll
        for (int e = 0; e < E; ++e) {
            const double q = base + e < P.Vs ? weight_of(qs, qrow, P.inv_t, base + e) / qs.total : 0.0;
            const double r = w[e] / ps.total - q;
            res[e] = r > 0.0 ? r : 0.0;
            s += res[e];
        }
        const double R = block_sum_d(s, sh);
        y = (R > 0.0) ? inv_cdf_row<E>(res, R, uf, sh) : inv_cdf_row<E>(w, ps.total, uf, sh);
    } else {
        y = inv_cdf_row<E>(w, ps.total, uf, sh);
    }
    }
    const int nb = n[b];
    for (int s2 = b; s2 < n_seq_streams; s2 += P.B) {
        const uint32_t* src = hid + ((size_t)s2 * (k + 1) + a) * hid_words;
        uint32_t* dst = hprev + (size_t)s2 * hid_words;
        for (int i = threadIdx.x; i < hid_words; i += NT) dst[i] = src[i];
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int i = 0; i < a; ++i) {
            const int t = draft[b * P.kstride + i];
            grid[(size_t)b * P.N + nb + i] = t;
            out_tok[b * (k + 1) + i] = t;
        }
        grid[(size_t)b * P.N + nb + a] = P.samp_lo + y;
        out_tok[b * (k + 1) + a] = P.samp_lo + y;
        out_na[b] = a;
        n[b] = nb + a + 1;
        atomicAdd(&counters[0], 1ull);
        atomicAdd(&counters[1], (unsigned long long)a);
        atomicAdd(&counters[2], (unsigned long long)(a + 1));
    }
}

// Several candidates at one position, each from a proposal of its own (Method, "Sampling and
// Verification", the recursion over consecutive rejections; appendix "Theoretical
// Justification", general form): p^(1) = p; candidate i is accepted iff u_i q_i(s_i) < p^(i)(s_i),
// otherwise p^(i+1) = norm(max(0, p^(i) - q_i)) (unchanged if that residual has no mass); after m
// rejections the token comes from p^(m+1) by inverse CDF.  One workgroup per position, the
// running target in registers (E fp64 values per thread), every proposal row read once.
// Candidates of a row: m, or the row's own count (clamped to 0 .. m) if the caller gives one.
__device__ __forceinline__ int row_candidates(const int32_t* m_rows, int row, int m) {
    return m_rows ? max(0, min(m, m_rows[row])) : m;
}

// Kept entries of a row gathered as scaled logits only (no indices): for the sum of their weights.
template <int E>
__device__ int compact_z(unsigned kmask, const float (&z)[E], float (&qz)[kCap], Shared& sh) {
    const int c = __popc(kmask);
    int at = block_excl_scan_i(c, sh);
    if (threadIdx.x == NT - 1) sh.b_int = at + c;
#pragma unroll
    for (int e = 0; e < E; ++e)
        if ((kmask >> e) & 1u) {
            if (at < kCap) qz[at] = z[e];
            ++at;
        }
    __syncthreads();
    return min(sh.b_int, kCap);
}

// The same recursion with the running target held as a list in LDS: top-k leaves at most kCap
// entries of p with mass, max(0, p - q) lives on those, and fp64 exponentials are evaluated for
// kept entries only, two per thread (the dense form spends one per vocabulary entry).
template <int E>
__global__ __launch_bounds__(NT) void multi_verify_list_kernel(const float* p_logits, const float* q_logits,
                                                               const int32_t* cand, const float* u_acc,
                                                               const float* u_final, const int32_t* m_rows, int m,
                                                               int n, float inv_t, int top_k, int32_t* out_index,
                                                               int32_t* out_token, double* out_resid) {
    __shared__ FastShared fs;
    __shared__ CompactList L;       // entries of p with mass: index, scaled logit, current p^(i)
    __shared__ float qz[kCap];      // kept scaled logits of the proposal at hand
    __shared__ double pick;
    const int row = blockIdx.x, i0 = threadIdx.x * 2;
    const int mr = row_candidates(m_rows, row, m);
    int Kp = 0, acc = mr, tok = -1;
    // One loop over the target row (i = -1) and the proposal rows, so that the top-k selection has
    // a single call site and is inlined with its LDS operands (a second copy would be called
    // through generic pointers).
    for (int i = -1; i < mr; ++i) {
        const float* qrow = i < 0 ? p_logits + (size_t)row * n : q_logits + ((size_t)row * m + i) * n;
        float z[E];
        unsigned km = 0u;
        load_row<E>(qrow, nullptr, 0.f, inv_t, nullptr, n, z);
        WarpStat qs = warp_select<E>(z, n, top_k, 0, fs, &km);
        if (i < 0) {   // p^(1): the kept entries of the target, normalised
            Kp = compact_row<E>(km, z, L, fs.sh);
            const double Zp = list_weights(L, Kp, qs.zmax, fs.sh);
#pragma unroll
            for (int e = 0; e < 2; ++e)
                if (i0 + e < Kp) L.w[i0 + e] /= Zp;   // the thread's own entries
            continue;
        }
        const int Kq = compact_z<E>(km, z, qz, fs.sh);
        double sq = 0.0;
#pragma unroll
        for (int e = 0; e < 2; ++e)
            if (i0 + e < Kq) sq += exp((double)qz[i0 + e] - (double)qs.zmax);
        if (threadIdx.x == 0) pick = 0.0;   // p^(i)(s) if s has no mass left
        qs.total = block_sum_d(sq, fs.sh);
        const int s_in = cand[(size_t)row * m + i];
        const bool s_ok = (unsigned)s_in < (unsigned)n;   // a token outside the slice is rejected, never read
        const int s = s_ok ? s_in : 0;
        double res[2], rs = 0.0;
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            res[e] = 0.0;
            if (i0 + e < Kp) {
                const int j = L.idx[i0 + e];
                const double pv = L.w[i0 + e];
                if (j == s) pick = pv;
                const double r = pv - weight_of(qs, qrow, inv_t, j) / qs.total;
                res[e] = r > 0.0 ? r : 0.0;
                rs += res[e];
            }
        }
        const double R = block_sum_d(rs, fs.sh);   // its barriers also publish pick
        const double pd = s_ok ? pick : 0.0, qd = s_ok ? weight_of(qs, qrow, inv_t, s) / qs.total : 1.0;
        if (out_resid && threadIdx.x == 0) out_resid[(size_t)row * m + i] = R;
        if ((double)u_acc[(size_t)row * m + i] * qd < pd) {
            acc = i;
            tok = s;
            break;
        }
        if (R > 0.0) {
#pragma unroll
            for (int e = 0; e < 2; ++e)
                if (i0 + e < Kp) L.w[i0 + e] = res[e] / R;
        }
    }
    if (acc == mr) {
        double sp = 0.0;
#pragma unroll
        for (int e = 0; e < 2; ++e)
            if (i0 + e < Kp) sp += L.w[i0 + e];
        const double total = block_sum_d(sp, fs.sh);
        tok = list_inv_cdf(L.w, L.idx, Kp, total, u_final[row], fs.sh);
    }
    if (threadIdx.x == 0) {
        out_index[row] = acc;
        out_token[row] = tok;
        if (out_resid)
            for (int i = (acc == mr ? mr : acc + 1); i < m; ++i) out_resid[(size_t)row * m + i] = -1.0;   // steps not evaluated
    }
}

// The same in two launches when the caller lends room for the rows' statistics: the top-k
// selection of the target row and of every proposal row runs in a workgroup of its own (all of
// them in parallel), and the walk over the candidates then only gathers.
template <int E>
__global__ __launch_bounds__(NT) void multi_row_stats_kernel(const float* p_logits, const float* q_logits,
                                                             const int32_t* m_rows, int m, int n, float inv_t,
                                                             int top_k, WarpStat* stats) {
    __shared__ FastShared fs;
    __shared__ CompactList L;
    const int j = blockIdx.x, row = blockIdx.y;   // j = 0: the target row, j >= 1: proposal j - 1
    if (j > row_candidates(m_rows, row, m)) return;
    const float* l = j == 0 ? p_logits + (size_t)row * n : q_logits + ((size_t)row * m + (j - 1)) * n;
    float z[E];
    load_row<E>(l, nullptr, 0.f, inv_t, nullptr, n, z);
    const WarpStat st = warp_and_draw<E>(z, n, top_k, 0, fs, L, nullptr, nullptr);
    if (threadIdx.x == 0) stats[(size_t)row * (m + 1) + j] = st;
}

template <int E>
__global__ __launch_bounds__(NT) void multi_verify_walk_kernel(const float* p_logits, const float* q_logits,
                                                               const int32_t* cand, const float* u_acc,
                                                               const float* u_final, const int32_t* m_rows, int m,
                                                               int n, float inv_t, const WarpStat* stats,
                                                               int32_t* out_index, int32_t* out_token,
                                                               double* out_resid) {
    __shared__ Shared sh;
    __shared__ CompactList L;       // entries of p with mass: index, scaled logit, current p^(i)
    __shared__ double pick;
    const int row = blockIdx.x, i0 = threadIdx.x * 2;
    const int mr = row_candidates(m_rows, row, m);
    const WarpStat ps = stats[(size_t)row * (m + 1)];
    float z[E];
    load_row<E>(p_logits + (size_t)row * n, nullptr, 0.f, inv_t, nullptr, n, z);
    const int Kp = compact_row<E>(kept_mask<E>(ps, z, n), z, L, sh);
    const double Zp = list_weights(L, Kp, ps.zmax, sh);
#pragma unroll
    for (int e = 0; e < 2; ++e)
        if (i0 + e < Kp) L.w[i0 + e] /= Zp;   // the thread's own entries
    int acc = mr, tok = -1;
    for (int i = 0; i < mr; ++i) {
        const float* qrow = q_logits + ((size_t)row * m + i) * n;
        const WarpStat qs = stats[(size_t)row * (m + 1) + 1 + i];
        const int s_in = cand[(size_t)row * m + i];
        const bool s_ok = (unsigned)s_in < (unsigned)n;   // a token outside the slice is rejected, never read
        const int s = s_ok ? s_in : 0;
        if (threadIdx.x == 0) pick = 0.0;   // p^(i)(s) if s has no mass left
        __syncthreads();
        double res[2], rs = 0.0;
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            res[e] = 0.0;
            if (i0 + e < Kp) {
                const int j = L.idx[i0 + e];
                const double pv = L.w[i0 + e];
                if (j == s) pick = pv;
                const double r = pv - weight_of(qs, qrow, inv_t, j) / qs.total;
                res[e] = r > 0.0 ? r : 0.0;
                rs += res[e];
            }
        }
        const double R = block_sum_d(rs, sh);   // its barriers also publish pick
        const double pd = s_ok ? pick : 0.0, qd = s_ok ? weight_of(qs, qrow, inv_t, s) / qs.total : 1.0;
        __syncthreads();   // pick is rewritten at the top of the next round
        if (out_resid && threadIdx.x == 0) out_resid[(size_t)row * m + i] = R;
        if ((double)u_acc[(size_t)row * m + i] * qd < pd) {
            acc = i;
            tok = s;
            break;
        }
        if (R > 0.0) {
#pragma unroll
            for (int e = 0; e < 2; ++e)
                if (i0 + e < Kp) L.w[i0 + e] = res[e] / R;
        }
    }
    if (acc == mr) {
        double sp = 0.0;
#pragma unroll
        for (int e = 0; e < 2; ++e)
            if (i0 + e < Kp) sp += L.w[i0 + e];
        const double total = block_sum_d(sp, sh);
        tok = list_inv_cdf(L.w, L.idx, Kp, total, u_final[row], sh);
    }
    if (threadIdx.x == 0) {
        out_index[row] = acc;
        out_token[row] = tok;
        if (out_resid)
            for (int i = (acc == mr ? mr : acc + 1); i < m; ++i) out_resid[(size_t)row * m + i] = -1.0;   // steps not evaluated
    }
}

template <int E>
__global__ __launch_bounds__(NT) void multi_verify_kernel(const float* p_logits, const float* q_logits,
                                                          const int32_t* cand, const float* u_acc,
                                                          const float* u_final, const int32_t* m_rows, int m, int n,
                                                          float inv_t, int top_k, int greedy, int32_t* out_index,
                                                          int32_t* out_token, double* out_resid) {
    __shared__ FastShared fs;
    __shared__ double pick[2];
    const int row = blockIdx.x, base = threadIdx.x * E;
    const int mr = row_candidates(m_rows, row, m);
    float z[E];
    unsigned km;
    load_row<E>(p_logits + (size_t)row * n, nullptr, 0.f, inv_t, nullptr, n, z);
    WarpStat ps = warp_select<E>(z, n, top_k, greedy, fs, &km);
    double p[E];
    dense_weights<E>(ps, z, p, fs.sh);
#pragma unroll
    for (int e = 0; e < E; ++e) p[e] /= ps.total;
    int acc = mr, tok = -1;
    for (int i = 0; i < mr; ++i) {
        if (threadIdx.x == 0) {   // a candidate outside the slice has no owner: p = 0, q = 1 rejects it
            pick[0] = 0.0;
            pick[1] = 1.0;
        }
        load_row<E>(q_logits + ((size_t)row * m + i) * n, nullptr, 0.f, inv_t, nullptr, n, z);
        WarpStat qs = warp_select<E>(z, n, top_k, greedy, fs, &km);
        double q[E];
        dense_weights<E>(qs, z, q, fs.sh);
        const int s = cand[(size_t)row * m + i];
        double rs = 0.0;
#pragma unroll
        for (int e = 0; e < E; ++e) {
            q[e] /= qs.total;
            if (base + e == s) {   // the owner of the candidate's entry publishes p^(i)(s), q_i(s)
                pick[0] = p[e];
                pick[1] = q[e];
            }
            const double r = p[e] - q[e];
            q[e] = r > 0.0 ? r : 0.0;   // q now holds max(0, p^(i) - q_i)
            rs += q[e];
        }
        const double R = block_sum_d(rs, fs.sh);   // its barriers also publish pick[]
        const double pd = pick[0], qd = pick[1];
        if (out_resid && threadIdx.x == 0) out_resid[(size_t)row * m + i] = R;
        const bool accept = (double)u_acc[(size_t)row * m + i] * qd < pd;
        __syncthreads();   // pick[] is rewritten by the next candidate
        if (accept) {
            acc = i;
            tok = s;
            break;
        }
        if (R > 0.0) {
#pragma unroll
            for (int e = 0; e < E; ++e) p[e] = q[e] / R;
        }
    }
    if (acc == mr) {
        double sp = 0.0;
#pragma unroll
        for (int e = 0; e < E; ++e) sp += p[e];
        const double total = block_sum_d(sp, fs.sh);
        tok = inv_cdf_row<E>(p, total, u_final[row], fs.sh);
    }
    if (threadIdx.x == 0) {
        out_index[row] = acc;
        out_token[row] = tok;
        if (out_resid)
            for (int i = (acc == mr ? mr : acc + 1); i < m; ++i) out_resid[(size_t)row * m + i] = -1.0;   // steps not evaluated
    }
}

// One draw per row from the row's warped distribution (inverse CDF over ascending index): the
// candidates of a sampling pool.  Rows whose entry of `skip` is negative give -1.
template <int E>
__global__ __launch_bounds__(NT) void sample_rows_kernel(const float* logits, const int32_t* skip, const float* u, int n,
                                                         float inv_t, int top_k, int greedy, int32_t* out_token) {
    __shared__ FastShared fs;
    __shared__ CompactList L;
    const int row = blockIdx.x;
    if (skip && skip[row] < 0) {
        if (threadIdx.x == 0) out_token[row] = -1;
        return;
    }
    float z[E];
    load_row<E>(logits + (size_t)row * n, nullptr, 0.f, inv_t, nullptr, n, z);
    const float ur = u[row];
    int drawn = 0;
    (void)warp_and_draw<E>(z, n, top_k, greedy, fs, L, &ur, &drawn);
    if (threadIdx.x == 0) out_token[row] = drawn;
}

SampParams samp_params(const hawk_ctx* c) {
    SampParams P;
    P.B = c->B; P.N = c->N; P.Vs = c->Vs; P.samp_lo = c->cfg.samp_lo; P.kstride = c->kmax + 1;
    P.top_k = c->top_k; P.greedy = c->greedy; P.use_cfg = c->cfg.use_cfg;
    P.inv_t = c->inv_t; P.cfg_scale = c->cfg_scale;
    return P;
}

}  // namespace

void launch_plan(hawk_ctx* c, int k) {
    plan_kernel<<<1, 64 * ((c->B + 63) / 64), 0, c->stream>>>(wsp<int32_t>(c, c->off.n), wsp<int32_t>(c, c->off.k_eff),
                                                            wsp<int32_t>(c, c->off.draft),
                                                            wsp<int32_t>(c, c->off.step),
                                                            wsp<unsigned long long>(c, c->off.counters), c->B, c->N,
                                                            k, c->kmax + 1);
}

// Entries per thread of the register-resident kernels for this vocabulary slice (0: too large).
static int fast_e(const hawk_ctx* c) { return c->Vs <= 4 * NT ? 4 : (c->Vs <= 16 * NT ? 16 : 0); }

void launch_first_token(hawk_ctx* c, const UniformSrc& us) {
    if (fast_e(c)) {
        auto kern = fast_e(c) == 4 ? first_token_fast<4> : first_token_fast<16>;
        kern<<<c->B, NT, 0, c->stream>>>(wsp<float>(c, c->off.logit_s), wsp<float>(c, c->off.logit_b),
                                         wsp<int32_t>(c, c->off.grid), wsp<int32_t>(c, c->off.n), samp_params(c), us);
        return;
    }
    first_token_kernel<<<c->B, NT, 0, c->stream>>>(wsp<float>(c, c->off.logit_s), wsp<float>(c, c->off.logit_b),
                                                   wsp<int32_t>(c, c->off.grid), wsp<int32_t>(c, c->off.n),
                                                   samp_params(c), us);
}

void launch_draft_sample(hawk_ctx* c, int i, int k, const UniformSrc& us, const DraftMode& dm) {
    ForcedSrc fs;
    fs.table = nullptr; fs.stride = 0; fs.relative = 0; fs.point_mass = dm.point_mass;
    if (dm.kind == 1) { fs.table = wsp<int32_t>(c, c->off.forced); fs.stride = k; }
    if (dm.kind == 2) { fs.table = wsp<int32_t>(c, c->off.replay); fs.stride = c->N; fs.relative = 1; }
    if (fast_e(c)) {
        auto kern = fast_e(c) == 4 ? draft_sample_fast<4> : draft_sample_fast<16>;
        kern<<<c->B, NT, 0, c->stream>>>(wsp<float>(c, c->off.dlogit_s), wsp<float>(c, c->off.dlogit_b),
                                         wsp<int32_t>(c, c->off.n), wsp<int32_t>(c, c->off.k_eff),
                                         wsp<int32_t>(c, c->off.draft), wsp<WarpStat>(c, c->off.qstat), i, k,
                                         samp_params(c), us, fs);
        return;
    }
    draft_sample_kernel<<<c->B, NT, 0, c->stream>>>(wsp<float>(c, c->off.dlogit_s), wsp<float>(c, c->off.dlogit_b),
                                                    wsp<int32_t>(c, c->off.n), wsp<int32_t>(c, c->off.k_eff),
                                                    wsp<int32_t>(c, c->off.draft), wsp<WarpStat>(c, c->off.qstat), i,
                                                    k, samp_params(c), us, fs);
}

void launch_verify_stats(hawk_ctx* c, int k) {
    if (fast_e(c)) {
        auto kern = fast_e(c) == 4 ? verify_stats_fast<4> : verify_stats_fast<16>;
        kern<<<dim3(k + 1, c->B), NT, 0, c->stream>>>(wsp<float>(c, c->off.logit_s), wsp<float>(c, c->off.logit_b),
                                                      wsp<int32_t>(c, c->off.k_eff), wsp<WarpStat>(c, c->off.pstat), k,
                                                      samp_params(c));
        return;
    }
    verify_stats_kernel<<<dim3(k + 1, c->B), NT, 0, c->stream>>>(
        wsp<float>(c, c->off.logit_s), wsp<float>(c, c->off.logit_b), wsp<int32_t>(c, c->off.k_eff),
        wsp<WarpStat>(c, c->off.pstat), k, samp_params(c));
}

void launch_accept_commit(hawk_ctx* c, int k, const UniformSrc& us) {
    if (fast_e(c)) {
        auto kern = fast_e(c) == 4 ? accept_commit_fast<4> : accept_commit_fast<16>;
        kern<<<c->B, NT, 0, c->stream>>>(
            wsp<float>(c, c->off.logit_b), wsp<float>(c, c->off.dlogit_b), wsp<WarpStat>(c, c->off.pstat),
            wsp<WarpStat>(c, c->off.qstat), wsp<int32_t>(c, c->off.k_eff), wsp<int32_t>(c, c->off.draft),
            wsp<int32_t>(c, c->off.grid), wsp<int32_t>(c, c->off.n), wsp<uint32_t>(c, c->off.x),
            wsp<uint32_t>(c, c->off.hprev), (int)(c->d * c->asz / 4), wsp<int32_t>(c, c->off.out_na),
            wsp<int32_t>(c, c->off.out_tok), wsp<unsigned long long>(c, c->off.counters), k, c->S, samp_params(c), us);
        return;
    }
    accept_commit_kernel<<<c->B, NT, 0, c->stream>>>(
        wsp<float>(c, c->off.logit_b), wsp<float>(c, c->off.dlogit_b), wsp<WarpStat>(c, c->off.pstat),
        wsp<WarpStat>(c, c->off.qstat), wsp<int32_t>(c, c->off.k_eff), wsp<int32_t>(c, c->off.draft),
        wsp<int32_t>(c, c->off.grid), wsp<int32_t>(c, c->off.n), wsp<uint32_t>(c, c->off.x),
        wsp<uint32_t>(c, c->off.hprev), (int)(c->d * c->asz / 4), wsp<int32_t>(c, c->off.out_na),
        wsp<int32_t>(c, c->off.out_tok), wsp<unsigned long long>(c, c->off.counters), k, c->S, samp_params(c), us);
}

void launch_force_setup(hawk_ctx* c, int cnt) {
    force_setup_kernel<<<1, 64 * ((c->B + 63) / 64), 0, c->stream>>>(
        wsp<int32_t>(c, c->off.u_draft), wsp<int32_t>(c, c->off.forced), wsp<int32_t>(c, c->off.n),
        wsp<int32_t>(c, c->off.k_eff), wsp<int32_t>(c, c->off.draft), c->B, cnt, c->kmax + 1);
}

void launch_force_commit(hawk_ctx* c, int cnt) {
    force_commit_kernel<<<c->B, 256, 0, c->stream>>>(wsp<int32_t>(c, c->off.forced), wsp<int32_t>(c, c->off.grid),
                                                     wsp<int32_t>(c, c->off.n), wsp<uint32_t>(c, c->off.x),
                                                     wsp<uint32_t>(c, c->off.hprev), (int)(c->d * c->asz / 4), c->B,
                                                     c->N, cnt, c->S);
}

int launch_sample_rows(const float* logits, const int32_t* skip, const float* u, int rows, int n, float temperature,
                       int top_k, int32_t* out_token, hipStream_t stream) {
    const int E = n <= 4 * NT ? 4 : (n <= 16 * NT ? 16 : 0);
    if (!E) return HAWK_EINVAL;
    const int greedy = (temperature == 0.0f || top_k == 1) ? 1 : 0;
    const float inv_t = greedy ? 1.0f : 1.0f / temperature;
    const int tk = top_k < n ? top_k : n;
    auto kern = E == 4 ? sample_rows_kernel<4> : sample_rows_kernel<16>;
    kern<<<rows, NT, 0, stream>>>(logits, skip, u, n, inv_t, tk, greedy, out_token);
    return hipGetLastError() == hipSuccess ? HAWK_OK : HAWK_EDEVICE;
}

size_t multi_verify_workspace_bytes(int rows, int m) { return (size_t)rows * (m + 1) * sizeof(WarpStat); }

int launch_multi_verify(const float* p_logits, const float* q_logits, const int32_t* cand, const float* u_acc,
                        const float* u_final, const int32_t* m_rows, int rows, int m, int n, float temperature, int top_k,
                        int32_t* out_index, int32_t* out_token, double* out_resid, void* workspace,
                        size_t workspace_bytes, hipStream_t stream) {
    const int E = n <= 4 * NT ? 4 : (n <= 16 * NT ? 16 : 0);
    if (!E) return HAWK_EINVAL;
    const int greedy = (temperature == 0.0f || top_k == 1) ? 1 : 0;
    const float inv_t = greedy ? 1.0f : 1.0f / temperature;
    const int tk = top_k < n ? top_k : n;
    if (use_list(tk, n, greedy) && workspace && workspace_bytes >= multi_verify_workspace_bytes(rows, m)) {
        WarpStat* stats = static_cast<WarpStat*>(workspace);
        auto k1 = E == 4 ? multi_row_stats_kernel<4> : multi_row_stats_kernel<16>;
        auto k2 = E == 4 ? multi_verify_walk_kernel<4> : multi_verify_walk_kernel<16>;
        k1<<<dim3(m + 1, rows), NT, 0, stream>>>(p_logits, q_logits, m_rows, m, n, inv_t, tk, stats);
        k2<<<rows, NT, 0, stream>>>(p_logits, q_logits, cand, u_acc, u_final, m_rows, m, n, inv_t, stats, out_index, out_token,
                                    out_resid);
    } else if (use_list(tk, n, greedy)) {
        auto kern = E == 4 ? multi_verify_list_kernel<4> : multi_verify_list_kernel<16>;
        kern<<<rows, NT, 0, stream>>>(p_logits, q_logits, cand, u_acc, u_final, m_rows, m, n, inv_t, tk, out_index, out_token,
                                      out_resid);
    } else {
        auto kern = E == 4 ? multi_verify_kernel<4> : multi_verify_kernel<16>;
        kern<<<rows, NT, 0, stream>>>(p_logits, q_logits, cand, u_acc, u_final, m_rows, m, n, inv_t, tk, greedy, out_index,
                                      out_token, out_resid);
    }
    return hipGetLastError() == hipSuccess ? HAWK_OK : HAWK_EDEVICE;
}

// ---- hawk_multi_verify for callers that cannot allocate: the rows' statistics live in a fixed array in
// device memory instead of a caller-provided workspace.  Every GPU holds its own copy of the array at
// its own address, looked up once per device; host code only ever uses that address.
constexpr int kStaticStatRows = 4096;   // logit rows (positions x (candidates + 1)) one call may have
static __device__ __align__(256) unsigned char scratch[(size_t)kStaticStatRows * sizeof(WarpStat)];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices];   // device address of `scratch` on each GPU (null: not looked up yet)

int scratch_address(void** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return HAWK_EDEVICE;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return HAWK_EDEVICE;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return HAWK_OK;
}
}  // namespace

int launch_multi_verify_static(const float* p_logits, const float* q_logits, const int32_t* cand, const float* u_acc,
                               const float* u_final, const int32_t* m_rows, int rows, int m, int n, float temperature,
                               int top_k, int32_t* out_index, int32_t* out_token, double* out_resid, hipStream_t stream) {
    if ((long long)rows * (m + 1) > kStaticStatRows) return HAWK_ENOMEM;
    void* ws = nullptr;
    const int rc = scratch_address(&ws);
    if (rc != HAWK_OK) return rc;
    // every record the second launch reads is written by the first launch of the same call, so
    // nothing in the array has to be cleared between calls
    return launch_multi_verify(p_logits, q_logits, cand, u_acc, u_final, m_rows, rows, m, n, temperature, top_k, out_index,
                               out_token, out_resid, ws, multi_verify_workspace_bytes(rows, m), stream);
}

}  // namespace hawk
