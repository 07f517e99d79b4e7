// spec_accept: accept / reject of drafted tokens with recovery or bonus token.
//
// Rule (Sec. 2.1 of the paper; the mismatch test and resampling distribution are those of
// speculative sampling): accept drafts while u * q(x) < p(x); at the first rejection draw
// one token from the normalised positive part of p - q; if everything is accepted and the
// call carries the extra target row, draw the bonus token from it.
//
// Work split.  A verification batch has few requests (16 .. 512) but a vocabulary of
// ~1.3e5, so one workgroup per request cannot fill the chip: every vocabulary row is cut
// into chunks of kChunk tokens and the vocabulary-wide sums are two-level.
//   stats    (LOGITS mode only) per row and group of 1-8 chunks: max of z / T and sum of exp(z / T - max) in
//            fp64.  A large call takes two passes: the rows the first kLazyJ drafts of every request need,
//            a first `decide` on those drafts, then the remaining rows of the requests still undecided and
//            `decide` once more for those (only rows 0 .. n of a request, n = accepted drafts, are needed)
//   decide   per request, one wave: the accept tests, one lane per draft with all gathers in flight
//            together; picks the row pair to sample from and records it
//   sample   grid (chunks, requests): every workgroup sums the fp64 mass of its chunk of the residual
//            and of the target row; the workgroup of a request that finishes last (found by an arrival
//            counter that `decide` has zeroed) draws the token: prefix over the chunk masses -> chunk
//            holding u * R -> scan inside that chunk
// Only the rows the outcome needs are streamed: one target row (bonus) or one target and
// one draft row (rejection) per request -- the algorithmic minimum in PROBS mode.
// All masses are accumulated in fp64 so that the chosen token matches a sequential fp64
// scan except when u * R lies within rounding of a CDF step.
#include <climits>

#include "common.hpp"
#include "device_utils.hpp"
#include "greedy_accept.hpp"

namespace fsr {
namespace {

constexpr int kChunk = 4096;        // vocabulary tokens per chunk
constexpr int kThreads = 256;       // threads per block in stats / partials / select
constexpr int kPerThread = kChunk / kThreads;  // 16 contiguous tokens per thread in select
constexpr int kMaxStatGroup = 8;    // LOGITS mode: most chunks whose softmax statistics one workgroup folds into one (max, sum) pair
constexpr int kLazyJ = 2;           // LOGITS mode, two-pass statistics: drafts tested before the rest of a request's rows is normalised
constexpr int kLazyMinRows = 3072;  // rows a call must be able to hold for the two extra launches of the two passes to pay
constexpr int kMaxSampleGroup = 8;  // accept_sample: a workgroup takes 1, 2, 4 or 8 consecutive chunks (see launch_all)
constexpr int kMaxChunksLds = 256;  // chunk masses of a request that the selecting workgroup keeps in LDS (vocabularies up to 2^20)

enum : int { kCaseNone = 0, kCaseResidual = 1, kCaseTarget = 2 };

// What `decide` hands to the later kernels, one per request.
struct Decision {
    long long t_row;  // storage row of the target distribution to sample from
    long long d_row;  // storage row of the draft distribution (residual case)
    double m_t, Z_t;  // LOGITS mode: max and partition sum of the target row
    double m_d, Z_d;  // ... of the draft row
    int kind;         // kCase*
    int n;            // accepted drafts
};

struct Workspace {
    Decision* dec;       // [B]
    double* mass_res;    // [B, n_chunks]
    double* mass_tgt;    // [B, n_chunks]
    double* stat_t;      // [R_t_cap, n_stat_groups, 2]  (LOGITS)
    double* stat_d;      // [R_d_cap, n_stat_groups, 2]
    unsigned int* arrivals;  // [B] chunk workgroups of the request that have finished (zeroed by decide)
    int stat_group;          // chunks per (max, sum) pair in this call (set at launch)
    int* pending;            // [B] (LOGITS, two-pass statistics) the request's first kLazyJ drafts were all accepted and more remain
};

__host__ __device__ inline int n_chunks_of(int V) { return (V + kChunk - 1) / kChunk; }
__host__ __device__ inline int n_stat_groups_of(int V, int group) { return (n_chunks_of(V) + group - 1) / group; }

size_t carve(const fsr_accept_params& p, char* base, Workspace* w) {
    const size_t nc = (size_t)n_chunks_of(p.V), B = (size_t)p.B;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        char* ptr = base ? base + off : nullptr;
        off += align_up(bytes, 256);
        return ptr;
    };
    Workspace tmp;
    tmp.dec = (Decision*)take(B * sizeof(Decision));
    tmp.mass_res = (double*)take(B * nc * sizeof(double));
    tmp.mass_tgt = (double*)take(B * nc * sizeof(double));
    tmp.arrivals = (unsigned int*)take(B * sizeof(unsigned int));
    tmp.pending = nullptr;
    tmp.stat_group = kMaxStatGroup;
    if (p.mode == FSR_LOGITS) {
        tmp.pending = (int*)take(B * sizeof(int));
        const size_t nsg = nc;  // room for one pair per chunk; a call folds 1, 2, 4 or 8 chunks into a pair
        tmp.stat_t = (double*)take(B * (size_t)(p.S_max + 1) * nsg * 2 * sizeof(double));
        tmp.stat_d = (double*)take(B * (size_t)p.S_max * nsg * 2 * sizeof(double));
    } else {
        tmp.stat_t = tmp.stat_d = nullptr;
    }
    if (w) *w = tmp;
    return off;
}

__device__ __forceinline__ double block_sum(double v, double* smem) {
    v = wave_sum(v);
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    __syncthreads();
    if (lane == 0) smem[w] = v;
    __syncthreads();
    double t = 0.0;
#pragma unroll
    for (int k = 0; k < kThreads / 64; ++k) t += smem[k];
    return t;
}

// Rows are fp32, or bf16 stored as 16-bit patterns (the upper half of an fp32).
__device__ __forceinline__ float to_float(float x) { return x; }
__device__ __forceinline__ float to_float(uint16_t x) { return __builtin_bit_cast(float, (uint32_t)x << 16); }
// May four consecutive values starting at a multiple of four be fetched with one vector load?
__device__ __forceinline__ bool row_vec_ok(const float* row) { return ((uintptr_t)row & 15) == 0; }
__device__ __forceinline__ bool row_vec_ok(const uint16_t* row) { return ((uintptr_t)row & 7) == 0; }

// Four consecutive values of a row starting at token e (bounds-checked: `fill` stands for tokens past the
// vocabulary; vector load when the row is aligned for it).
__device__ __forceinline__ void load_quad(const float* __restrict__ row, int e, int V, bool vec, float (&x)[4],
                                          float fill = 0.0f) {
    if (vec && e + 3 < V) {
        const float4 t = *reinterpret_cast<const float4*>(row + e);
        x[0] = t.x; x[1] = t.y; x[2] = t.z; x[3] = t.w;
    } else {
#pragma unroll
        for (int k = 0; k < 4; ++k) x[k] = (e + k < V) ? row[e + k] : fill;
    }
}
__device__ __forceinline__ void load_quad(const uint16_t* __restrict__ row, int e, int V, bool vec, float (&x)[4],
                                          float fill = 0.0f) {
    if (vec && e + 3 < V) {
        const uint2 t = *reinterpret_cast<const uint2*>(row + e);
        x[0] = __builtin_bit_cast(float, t.x << 16);
        x[1] = __builtin_bit_cast(float, t.x & 0xffff0000u);
        x[2] = __builtin_bit_cast(float, t.y << 16);
        x[3] = __builtin_bit_cast(float, t.y & 0xffff0000u);
    } else {
#pragma unroll
        for (int k = 0; k < 4; ++k) x[k] = (e + k < V) ? to_float(row[e + k]) : fill;
    }
}

// The same where the caller has checked that the row is aligned and the four tokens exist: the load and nothing else.
__device__ __forceinline__ void load_quad_vec(const float* __restrict__ row, int e, float (&x)[4]) {
    const float4 t = *reinterpret_cast<const float4*>(row + e);
    x[0] = t.x; x[1] = t.y; x[2] = t.z; x[3] = t.w;
}
__device__ __forceinline__ void load_quad_vec(const uint16_t* __restrict__ row, int e, float (&x)[4]) {
    const uint2 t = *reinterpret_cast<const uint2*>(row + e);
    x[0] = __builtin_bit_cast(float, t.x << 16);
    x[1] = __builtin_bit_cast(float, t.x & 0xffff0000u);
    x[2] = __builtin_bit_cast(float, t.y << 16);
    x[3] = __builtin_bit_cast(float, t.y & 0xffff0000u);
}

// Constants of exp_softmax, made once per kernel.  The empty asm statements pin each one to a scalar register pair
// (the leading coefficient to a vector pair) and hide its value from the compiler, which otherwise rebuilds every
// constant with move instructions in front of each use: that doubles the instruction count of the polynomial.
struct ExpConsts {
    double floor, log2e, nln2_hi, nln2_lo, magic, c10, c9, c8, c7, c6, c5, c4, c3, c2, c1;
};
__device__ __forceinline__ ExpConsts exp_consts() {
    ExpConsts k;
    k.floor = -800.0;  // below it exp is 0 in fp64
    k.log2e = 1.4426950408889634074;
    k.nln2_hi = -6.93147180369123816490e-01;  // high part of ln2: its last 21 bits are zero, so k * hi is exact for |k| < 2^21
    k.nln2_lo = -1.90821492927058770002e-10;
    k.magic = 6755399441055744.0;  // 1.5 * 2^52: adding it rounds to an integer and leaves that integer in the low word
    // the polynomial of degree 10 that equals exp at the 11 Chebyshev nodes of [-ln2/2, ln2/2] (widened by 0.05 %),
    // solved in 80-bit arithmetic and rounded to fp64: 3e-16 from exp over the interval, 5e-16 as evaluated
    k.c10 = 2.7626457017679406e-07;
    k.c9 = 2.7640263805714195e-06;
    k.c8 = 2.480150410776298e-05;
    k.c7 = 0.00019841170070855952;
    k.c6 = 0.0013888888932672718;
    k.c5 = 0.008333333385825259;
    k.c4 = 0.041666666666572656;
    k.c3 = 0.16666666666553953;
    k.c2 = 0.5000000000000006;
    k.c1 = 1.0000000000000069;
    asm volatile("" : "+s"(k.log2e), "+s"(k.nln2_hi), "+s"(k.nln2_lo), "+s"(k.floor), "+v"(k.c10), "+v"(k.magic));
    asm volatile("" : "+s"(k.c9), "+s"(k.c8), "+s"(k.c7), "+s"(k.c6), "+s"(k.c5));
    asm volatile("" : "+s"(k.c4), "+s"(k.c3), "+s"(k.c2), "+s"(k.c1));
    return k;
}

// exp(x) in fp64 for the arguments a softmax produces (x <= 0 after the row maximum is taken off; x up to a few
// hundred works too; x below -745, -inf included, gives 0, and so does NaN: such a logit counts as masked).
// x = k ln2 + r with |r| <= ln2 / 2: k by adding 1.5 * 2^52 to x log2(e), which rounds to the integer and leaves it
// in the sum's low word; ln2 in two parts so that r is exact to the last bit; exp(r) by a polynomial of degree 10
// (5e-16 relative); times 2^k by ldexp, which also makes the subnormal results and the final 0.  16 instructions,
// all of them issued at the full fp64 rate, where the library routine takes several times as many: the per-element
// exp is what bounds the LOGITS-mode kernels.
__device__ __forceinline__ double exp_softmax(double x, const ExpConsts& k) {
    x = fmax(x, k.floor);
    const double t = fma(x, k.log2e, k.magic);
    const double kf = t - k.magic;
    double r = fma(kf, k.nln2_hi, x);
    r = fma(kf, k.nln2_lo, r);
    double p = fma(k.c10, r, k.c9);
    p = fma(p, r, k.c8);
    p = fma(p, r, k.c7);
    p = fma(p, r, k.c6);
    p = fma(p, r, k.c5);
    p = fma(p, r, k.c4);
    p = fma(p, r, k.c3);
    p = fma(p, r, k.c2);
    p = fma(p, r, k.c1);
    p = fma(p, r, 1.0);
    return ldexp(p, (int)(uint32_t)__builtin_bit_cast(unsigned long long, t));
}
// The constants for a kernel of the given mode: PROBS mode never evaluates exp and gets an empty set.
template <int MODE>
__device__ __forceinline__ ExpConsts exp_consts_for() {
    if constexpr (MODE == FSR_LOGITS) return exp_consts();
    else return ExpConsts{};
}

// Probability of one entry in fp64: the value itself, or exp(z / T - m) / Z with the two divisions as products
// by 1 / T and 1 / Z (loop invariants the compiler hoists).  m is a maximum of values z * (1 / T) formed the same
// way, so the row's largest entry gives exp(0) exactly.
template <int MODE>
__device__ __forceinline__ double prob_of(float x, double T, double m, double Z, const ExpConsts& ek) {
    if constexpr (MODE == FSR_PROBS) {
        return (double)x;
    } else {
        return exp_softmax((double)x * (1.0 / T) - m, ek) * (1.0 / Z);
    }
}

// ---------------------------------------------------------------------------------------
// LOGITS mode: per row and group of ws.stat_group chunks, the maximum of z / T and the sum of exp(z / T - max), fp64.
// grid = (n_stat_groups, B * slots): a request owns `slots` consecutive workgroup rows; slot k < t_n is its target
// row t_lo + k, the others are its draft rows d_lo, d_lo + 1, ...  (which of the request's rows a pass covers is
// the host's choice: all of them, those of the first kLazyJ drafts, or the rest for the requests left pending).
// Each lane keeps a running maximum and a sum relative to it over its own elements (16 per chunk), so the chunks of
// a group need no exchange between lanes; lanes and waves are combined once, at the end.
// ---------------------------------------------------------------------------------------
template <typename RT>
__global__ __launch_bounds__(kThreads) void accept_stats_kernel(
    const RT* __restrict__ z_target, const RT* __restrict__ z_draft, const int32_t* __restrict__ cu_t,
    const int32_t* __restrict__ cu_d, const int32_t* __restrict__ t_rows, const int32_t* __restrict__ d_rows,
    Workspace ws, int B, int V, int S_max, double T, int slots, int t_lo, int t_n, int d_lo, int only_pending) {
    __shared__ double s_sum[kThreads / 64];
    __shared__ float s_max[kThreads / 64];
    const int nc = n_chunks_of(V), nsg = n_stat_groups_of(V, ws.stat_group);
    const int i = blockIdx.y / slots, k = blockIdx.y - i * slots;
    if (only_pending && !ws.pending[i]) return;
    const RT* rows;
    double* stat;
    if (k < t_n) {
        const int j = t_lo + k, t0 = cu_t[i], t_i = cu_t[i + 1] - t0;
        const long long r = (long long)t0 + j;
        // no such row, or past what the workspace or the caller's row map holds (offsets of an invalid call)
        if (j >= t_i || t0 < 0 || r >= (long long)B * (S_max + 1) || r >= cu_t[B]) return;
        rows = z_target + (size_t)(t_rows ? t_rows[r] : r) * V;
        stat = ws.stat_t + ((size_t)r * nsg + blockIdx.x) * 2;
    } else {
        const int j = d_lo + (k - t_n), d0 = cu_d[i], d_i = cu_d[i + 1] - d0;
        const long long r = (long long)d0 + j;
        if (j >= d_i || d0 < 0 || r >= (long long)B * S_max || r >= cu_d[B]) return;
        rows = z_draft + (size_t)(d_rows ? d_rows[r] : r) * V;
        stat = ws.stat_d + ((size_t)r * nsg + blockIdx.x) * 2;
    }
    const bool vec = row_vec_ok(rows);
    const double inv_T = 1.0 / T;
    const ExpConsts ek = exp_consts();
    const int c_first = blockIdx.x * ws.stat_group, c_end = min(nc, c_first + ws.stat_group);
    float mz = -INFINITY;  // largest logit this lane has seen
    double mzT = 0.0;      // mz / T once mz is finite
    double sum = 0.0;      // sum of exp(z / T - mz / T) over this lane's elements
    // The fold over the group's chunks, twice: for whole chunks of a row aligned for vector loads (four loads per
    // lane and chunk, all in flight together, the next chunk's issued before this one's arithmetic), and with every
    // element bounds-checked for the chunk that holds the vocabulary's ragged end or a row that is not aligned.
    // Two separate loops, because mixed in one the compiler orders each vector load behind all loads before it.
    auto fold = [&](auto whole, int c_lo, int c_hi) {
        float cur[kPerThread], nxt[kPerThread];
        auto load_chunk = [&](int c, float (&v)[kPerThread]) {
#pragma unroll
            for (int q = 0; q < kPerThread / 4; ++q) {
                float x[4];
                const int e = c * kChunk + (q * kThreads + threadIdx.x) * 4;
                if constexpr (decltype(whole)::value) load_quad_vec(rows, e, x);
                else load_quad(rows, e, V, vec, x, -INFINITY);
#pragma unroll
                for (int u = 0; u < 4; ++u) v[q * 4 + u] = x[u];
            }
        };
        if (c_lo >= c_hi) return;
        load_chunk(c_lo, cur);
        for (int c = c_lo; c < c_hi; ++c) {
            if (c + 1 < c_hi) load_chunk(c + 1, nxt);
            float mx = cur[0];
#pragma unroll
            for (int u = 1; u < kPerThread; ++u) mx = fmaxf(mx, cur[u]);
            if (mx > mz) {  // rescale what was summed against the old maximum
                const double mxT = (double)mx * inv_T;
                sum = mz == -INFINITY ? 0.0 : sum * exp_softmax(mzT - mxT, ek);
                mz = mx;
                mzT = mxT;
            }
#pragma unroll
            for (int u = 0; u < kPerThread; ++u) sum += exp_softmax((double)cur[u] * inv_T - mzT, ek);  // -inf (masked, or past V) adds 0
#pragma unroll
            for (int u = 0; u < kPerThread; ++u) cur[u] = nxt[u];
        }
    };
    const int c_whole = vec ? min(c_end, V / kChunk) : c_first;  // chunks before it are whole and aligned
    fold(std::true_type{}, c_first, c_whole);
    fold(std::false_type{}, max(c_first, c_whole), c_end);
    // lanes -> wave -> workgroup, each time against the common maximum
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const float mw = wave_max(mz);
    sum = mz == -INFINITY ? 0.0 : sum * exp_softmax(mzT - (double)mw * inv_T, ek);
    sum = wave_sum(sum);
    if (lane == 0) {
        s_max[w] = mw;
        s_sum[w] = sum;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        const float mg = fmaxf(fmaxf(s_max[0], s_max[1]), fmaxf(s_max[2], s_max[3]));
        const double mgT = (double)mg * inv_T;
        double tot = 0.0;
#pragma unroll
        for (int q = 0; q < kThreads / 64; ++q)
            if (s_max[q] != -INFINITY) tot += s_sum[q] * exp_softmax((double)s_max[q] * inv_T - mgT, ek);
        stat[0] = mgT;  // -inf for a group of masked logits only
        stat[1] = tot;
    }
}

// Combine a row's chunk statistics into (max, partition sum); all lanes of the wave call it.
__device__ __forceinline__ void combine_stats(const double* __restrict__ stat, int nc, const ExpConsts& ek, double& m, double& Z) {
    const int lane = threadIdx.x & 63;
    double mm = -INFINITY;
    for (int c = lane; c < nc; c += 64) mm = fmax(mm, stat[c * 2]);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mm = fmax(mm, __shfl_xor(mm, o, 64));
    double z = 0.0;
    for (int c = lane; c < nc; c += 64) z += stat[c * 2 + 1] * exp_softmax(stat[c * 2] - mm, ek);
    m = mm;
    Z = wave_sum(z);
}
// The same by one lane on its own (every lane of the wave works on a different row): the pairs four at a time, all
// eight loads of a batch in flight together, folded with a running maximum.
__device__ __forceinline__ void combine_stats_lane(const double* __restrict__ stat, int nc, const ExpConsts& ek, double& m,
                                                   double& Z) {
    double mm = -INFINITY, z = 0.0;
    for (int c0 = 0; c0 < nc; c0 += 4) {
        double mc[4], sc[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int c = min(c0 + u, nc - 1);
            mc[u] = stat[c * 2];
            sc[u] = stat[c * 2 + 1];
        }
        double mb = mc[0];
#pragma unroll
        for (int u = 1; u < 4; ++u) mb = fmax(mb, c0 + u < nc ? mc[u] : -INFINITY);
        if (mb > mm) {
            z = mm == -INFINITY ? 0.0 : z * exp_softmax(mm - mb, ek);
            mm = mb;
        }
        if (mm != -INFINITY) {
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (c0 + u < nc) z += sc[u] * exp_softmax(mc[u] - mm, ek);
        }
    }
    m = mm;
    Z = z;
}

// Masses of 4 consecutive tokens starting at e for the request's decision (bounds-checked).
template <int MODE, typename RT>
__device__ __forceinline__ void quad_masses(const Decision& dec, const RT* __restrict__ trow,
                                            const RT* __restrict__ drow, int e, int V, bool vec_t, bool vec_d,
                                            double T, const ExpConsts& ek, double (&res)[4], double (&tgt)[4]) {
    float a[4], b[4];
    load_quad(trow, e, V, vec_t, a);
    if (dec.kind == kCaseResidual) load_quad(drow, e, V, vec_d, b);
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const bool ok = e + k < V;
        const double pt = ok ? prob_of<MODE>(a[k], T, dec.m_t, dec.Z_t, ek) : 0.0;
        tgt[k] = pt;
        if (dec.kind == kCaseResidual) {
            const double qd = ok ? prob_of<MODE>(b[k], T, dec.m_d, dec.Z_d, ek) : 0.0;
            const double r = pt - qd;
            res[k] = r > 0.0 ? r : 0.0;
        } else {
            res[k] = pt;
        }
    }
}

__device__ __forceinline__ double shfl_f64(double v, int src) {
    const unsigned long long b = __builtin_bit_cast(unsigned long long, v);
    const uint32_t lo = __shfl((uint32_t)b, src, 64), hi = __shfl((uint32_t)(b >> 32), src, 64);
    return __builtin_bit_cast(double, ((unsigned long long)hi << 32) | lo);
}
__device__ __forceinline__ long long shfl_i64(long long v, int src) {
    const uint32_t lo = __shfl((uint32_t)v, src, 64), hi = __shfl((uint32_t)((unsigned long long)v >> 32), src, 64);
    return (long long)(((unsigned long long)hi << 32) | lo);
}
// 8-byte values that another workgroup of the same launch reads: stored through to memory / loaded past the caches
__device__ __forceinline__ void publish_f64(double* p, double v) {
    __hip_atomic_store(reinterpret_cast<unsigned long long*>(p), __builtin_bit_cast(unsigned long long, v), __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ double fetch_f64(const double* p) {
    return __builtin_bit_cast(double, __hip_atomic_load(reinterpret_cast<const unsigned long long*>(p), __ATOMIC_RELAXED,
                                                         __HIP_MEMORY_SCOPE_AGENT));
}

// ---------------------------------------------------------------------------------------
// decide: one wave per request; lane n tests draft n.
// ---------------------------------------------------------------------------------------
// PHASE 0: all drafts.  PHASE 1 (LOGITS, two-phase statistics): only the first kLazyJ drafts; a request whose first
// kLazyJ drafts are all accepted and that has more is left pending, everything else is final.  PHASE 2: the pending
// requests, from the start, now that all their rows are normalised.
template <int MODE, typename RT, int PHASE>
__global__ __launch_bounds__(64) void accept_decide_kernel(
    const RT* __restrict__ p_target, const RT* __restrict__ p_draft, const int32_t* __restrict__ draft_tokens,
    const float* __restrict__ u_accept, const int32_t* __restrict__ cu_t, const int32_t* __restrict__ cu_d,
    const int32_t* __restrict__ t_rows, const int32_t* __restrict__ d_rows, int32_t* __restrict__ accepted_len,
    int32_t* __restrict__ n_emitted, int32_t* __restrict__ emitted, Workspace ws, int B, int V, int S_max, double T) {
    const int i = blockIdx.x, lane = threadIdx.x;
    if (PHASE == 2 && !ws.pending[i]) return;
    const int nsg = n_stat_groups_of(V, ws.stat_group);
    const int t0 = cu_t[i], t_i = cu_t[i + 1] - t0, d0 = cu_d[i], d_i = cu_d[i + 1] - d0;
    int32_t* em = emitted + (size_t)i * (S_max + 1);
    Decision dec;
    dec.kind = kCaseNone;
    dec.n = 0;
    dec.t_row = dec.d_row = 0;
    dec.m_t = dec.m_d = 0.0;
    dec.Z_t = dec.Z_d = 1.0;
    if (lane == 0) ws.arrivals[i] = 0u;
    // the per-row statistics hold B*(S_max+1) target and B*S_max draft rows: a call whose offsets
    // run past that (only possible after an invalid request) is refused for the requests beyond
    const bool fits = (long long)t0 + t_i <= (long long)B * (S_max + 1) && (long long)d0 + d_i <= (long long)B * S_max;
    if (d_i < 0 || d_i > S_max || t_i < d_i || t_i > d_i + 1 || t0 < 0 || d0 < 0 || !fits) {
        for (int s = lane; s <= S_max; s += 64) em[s] = -1;
        if (lane == 0) {
            accepted_len[i] = -1;
            n_emitted[i] = -1;
            ws.dec[i] = dec;
            if (PHASE == 1) ws.pending[i] = 0;
        }
        return;
    }
    const int d_lim = PHASE == 1 ? min(d_i, kLazyJ) : d_i;  // drafts this pass tests
    const ExpConsts ek = exp_consts_for<MODE>();
    int n = d_lim;  // accepted drafts
    for (int n0 = 0; n0 < d_lim && n == d_lim; n0 += 64) {
        const int k = n0 + lane;
        const bool live = k < d_lim;
        long long tr = 0, dr = 0;
        double m_t = 0.0, Z_t = 1.0, m_d = 0.0, Z_d = 1.0;
        int x = 0;
        bool ok = true;
        if (live) {
            tr = t_rows ? t_rows[t0 + k] : t0 + k;
            dr = d_rows ? d_rows[d0 + k] : d0 + k;
            x = min(max(draft_tokens[dr], 0), V - 1);
            const double u = (double)u_accept[dr];
            if constexpr (MODE == FSR_LOGITS) {
                combine_stats_lane(ws.stat_t + (size_t)(t0 + k) * nsg * 2, nsg, ek, m_t, Z_t);
                combine_stats_lane(ws.stat_d + (size_t)(d0 + k) * nsg * 2, nsg, ek, m_d, Z_d);
            }
            const double px = prob_of<MODE>(to_float(p_target[(size_t)tr * V + x]), T, m_t, Z_t, ek);
            const double qx = prob_of<MODE>(to_float(p_draft[(size_t)dr * V + x]), T, m_d, Z_d, ek);
            ok = u * qx < px;
        }
        const unsigned long long rejected = __builtin_amdgcn_ballot_w64(live && !ok);
        const int first = rejected ? (int)__builtin_ctzll(rejected) : 64;
        if (live && lane < first) em[k] = x;  // accepted drafts of this round of 64
        if (rejected) {
            n = n0 + first;
            dec.kind = kCaseResidual;
            dec.t_row = shfl_i64(tr, first);
            dec.d_row = shfl_i64(dr, first);
            dec.m_t = shfl_f64(m_t, first); dec.Z_t = shfl_f64(Z_t, first);
            dec.m_d = shfl_f64(m_d, first); dec.Z_d = shfl_f64(Z_d, first);
        }
    }
    if (PHASE == 1) {
        const bool pending = n == d_lim && d_i > d_lim;  // nothing rejected so far and drafts remain
        if (lane == 0) ws.pending[i] = pending ? 1 : 0;
        if (pending) return;
    }
    dec.n = n;
    if (n == d_i && t_i == d_i + 1) {
        dec.kind = kCaseTarget;
        dec.t_row = t_rows ? t_rows[t0 + d_i] : t0 + d_i;
        if constexpr (MODE == FSR_LOGITS) combine_stats(ws.stat_t + (size_t)(t0 + d_i) * nsg * 2, nsg, ek, dec.m_t, dec.Z_t);
    }
    for (int s = n + lane; s <= S_max; s += 64) em[s] = -1;
    if (lane == 0) {
        accepted_len[i] = n;
        n_emitted[i] = n;  // the sampling kernel adds the drawn token
        ws.dec[i] = dec;
    }
}

// ---------------------------------------------------------------------------------------
// sample: request i = blockIdx.y; this workgroup owns chunks kSampleGroup * blockIdx.x .. + kSampleGroup - 1 of the
// vocabulary.  grid = (ceil(n_chunks / kSampleGroup), B)
// ---------------------------------------------------------------------------------------
template <int MODE, typename RT, int kSampleGroup>
__global__ __launch_bounds__(kThreads) void accept_sample_kernel(
    const RT* __restrict__ p_target, const RT* __restrict__ p_draft, const float* __restrict__ u_sample,
    int32_t* __restrict__ n_emitted, int32_t* __restrict__ emitted, Workspace ws, int V, int S_max, double T) {
    __shared__ double s_part[kThreads / 64][2 * kSampleGroup];
    __shared__ double s_wave[kThreads / 64];
    __shared__ int s_i[kThreads / 64];
    __shared__ double s_base, s_thr;
    __shared__ int s_chunk, s_fallback, s_last;
    __shared__ double s_mass[2 * kMaxChunksLds];
    const int nc = n_chunks_of(V), i = blockIdx.y;
    const ExpConsts ek = exp_consts_for<MODE>();
    const int c_first = blockIdx.x * kSampleGroup, n_here = min(kSampleGroup, nc - c_first);
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    int32_t* em = emitted + (size_t)i * (S_max + 1);
    Decision dec = ws.dec[i];
    dec.kind = __builtin_amdgcn_readfirstlane(dec.kind);  // the same in every lane: say so, branches on it stay scalar
    if (dec.kind == kCaseNone) return;

    // ---- 2. fp64 mass of this chunk of the sampling distribution (and of the target row, for the fallback)
    const RT* trow = p_target + (size_t)dec.t_row * V;
    const RT* drow = p_draft + (size_t)dec.d_row * V;
    const bool vec_t = row_vec_ok(trow), vec_d = row_vec_ok(drow);
    // A workgroup takes kSampleGroup consecutive chunks: the chain every workgroup goes through (decision record,
    // row loads, reduction, store-through, arrival count) is paid once per 128 KB instead of once per 32 KB.  Each
    // chunk's mass is reduced exactly as if it had a workgroup to itself (thread sums, wave sums, waves in order).
    {
        // whole chunks of aligned rows first, through code that has only vector loads (the next chunk's issued before
        // this chunk's arithmetic); then the chunk with the vocabulary's ragged end (or every chunk, if a row is not
        // aligned), bounds-checked.  A chunk's two masses go to LDS as soon as the wave has them.
        const bool vec_ok = vec_t && (dec.kind != kCaseResidual || vec_d);
        const int n_whole = vec_ok ? min(n_here, max(0, V / kChunk - c_first)) : 0;
        const bool residual = dec.kind == kCaseResidual;
        if (n_whole > 0) {
            float ta[kPerThread], da[kPerThread], tb[kPerThread], db[kPerThread];
            auto load_rows = [&](int c, float (&t)[kPerThread], float (&d)[kPerThread]) {
#pragma unroll
                for (int k = 0; k < kPerThread / 4; ++k) {
                    const int e = c * kChunk + (k * kThreads + threadIdx.x) * 4;
                    float x[4], y[4] = {0.0f, 0.0f, 0.0f, 0.0f};
                    load_quad_vec(trow, e, x);
                    if (residual) load_quad_vec(drow, e, y);
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        t[4 * k + u] = x[u];
                        d[4 * k + u] = y[u];
                    }
                }
            };
            load_rows(c_first, ta, da);
            for (int cc = 0; cc < n_whole; ++cc) {
                if (cc + 1 < n_whole) load_rows(c_first + cc + 1, tb, db);
                double r = 0.0, t = 0.0;
#pragma unroll
                for (int k = 0; k < kPerThread / 4; ++k) {
                    double res[4], tgt[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const double pt = prob_of<MODE>(ta[4 * k + u], T, dec.m_t, dec.Z_t, ek);
                        tgt[u] = pt;
                        if (residual) {
                            const double d = pt - prob_of<MODE>(da[4 * k + u], T, dec.m_d, dec.Z_d, ek);
                            res[u] = d > 0.0 ? d : 0.0;
                        } else {
                            res[u] = pt;
                        }
                    }
                    r += (res[0] + res[1]) + (res[2] + res[3]);
                    t += (tgt[0] + tgt[1]) + (tgt[2] + tgt[3]);
                }
                r = wave_sum(r);
                t = wave_sum(t);
                if (lane == 0) {
                    s_part[w][2 * cc] = r;
                    s_part[w][2 * cc + 1] = t;
                }
#pragma unroll
                for (int u = 0; u < kPerThread; ++u) {
                    ta[u] = tb[u];
                    da[u] = db[u];
                }
            }
        }
#pragma unroll 1
        for (int cs = n_whole; cs < n_here; ++cs) {
            const int e0 = (c_first + cs) * kChunk;
            double r = 0.0, t = 0.0;
#pragma unroll
            for (int k = 0; k < kPerThread / 4; ++k) {
                const int e = e0 + (k * kThreads + threadIdx.x) * 4;
                double res[4], tgt[4];
                quad_masses<MODE, RT>(dec, trow, drow, e, V, vec_t, vec_d, T, ek, res, tgt);
                r += (res[0] + res[1]) + (res[2] + res[3]);
                t += (tgt[0] + tgt[1]) + (tgt[2] + tgt[3]);
            }
            r = wave_sum(r);
            t = wave_sum(t);
            if (lane == 0) {
                s_part[w][2 * cs] = r;
                s_part[w][2 * cs + 1] = t;
            }
        }
        __syncthreads();
        if (threadIdx.x == 0) {
            for (int cc = 0; cc < n_here; ++cc) {
                double tr = 0.0, tt = 0.0;
#pragma unroll
                for (int k = 0; k < kThreads / 64; ++k) {
                    tr += s_part[k][2 * cc];
                    tt += s_part[k][2 * cc + 1];
                }
                publish_f64(ws.mass_res + (size_t)i * nc + c_first + cc, tr);
                publish_f64(ws.mass_tgt + (size_t)i * nc + c_first + cc, tt);
            }
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // all are in memory before the arrivals are counted
            s_last = atomicAdd(ws.arrivals + i, (unsigned)n_here) + (unsigned)n_here == (unsigned)nc;
        }
        __syncthreads();
        if (!s_last) return;
    }

    // ---- 3. the request's last workgroup draws the token: total mass and the chunk that holds u * R.
    // The chunk masses come from memory (other workgroups wrote them): all threads fetch them together
    // into LDS, then one thread runs the sequential fp64 prefix over the <= a few dozen chunks.
    double* l_res = reinterpret_cast<double*>(s_mass);
    double* l_tgt = l_res + kMaxChunksLds;
    const bool in_lds = nc <= kMaxChunksLds;
    if (in_lds) {
        for (int cc = threadIdx.x; cc < nc; cc += kThreads) {
            l_res[cc] = fetch_f64(ws.mass_res + (size_t)i * nc + cc);
            l_tgt[cc] = fetch_f64(ws.mass_tgt + (size_t)i * nc + cc);
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        const double* gres = ws.mass_res + (size_t)i * nc;
        const double* gtgt = ws.mass_tgt + (size_t)i * nc;
        auto mres = [&](int cc) { return in_lds ? l_res[cc] : fetch_f64(gres + cc); };
        auto mtgt = [&](int cc) { return in_lds ? l_tgt[cc] : fetch_f64(gtgt + cc); };
        double R = 0.0;
        for (int cc = 0; cc < nc; ++cc) R += mres(cc);
        int fallback = 0;
        if (!(R > 0.0)) {  // residual is all zero: sample from the target row itself
            fallback = 1;
            R = 0.0;
            for (int cc = 0; cc < nc; ++cc) R += mtgt(cc);
        }
        const double thr = (double)u_sample[i] * R;
        double acc = 0.0, base = 0.0;
        int chunk = -1, last_pos = 0;
        double last_base = 0.0;
        for (int cc = 0; cc < nc; ++cc) {
            const double prev = acc, mc = fallback ? mtgt(cc) : mres(cc);
            acc += mc;
            if (mc > 0.0) {
                last_pos = cc;
                last_base = prev;
                if (acc > thr) {
                    chunk = cc;
                    base = prev;
                    break;
                }
            }
        }
        if (chunk < 0) {  // rounding left no chunk: the last chunk with mass
            chunk = last_pos;
            base = last_base;
        }
        s_base = base;
        s_thr = thr;
        s_chunk = chunk;
        s_fallback = fallback;
    }
    __syncthreads();
    if (s_fallback) dec.kind = kCaseTarget;
    const double thr = s_thr;
    const int cs = s_chunk;

    // scan inside the chunk: thread t owns tokens [16 t, 16 t + 16) of the chunk
    const int e0 = cs * kChunk + threadIdx.x * kPerThread;
    double mass[kPerThread];
    double local = 0.0;
#pragma unroll
    for (int k = 0; k < kPerThread / 4; ++k) {
        double res[4], tgt[4];
        quad_masses<MODE, RT>(dec, trow, drow, e0 + 4 * k, V, vec_t, vec_d, T, ek, res, tgt);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            mass[4 * k + j] = res[j];
            local += res[j];
        }
    }
    const double inc = wave_inclusive_scan(local);
    if (lane == 63) s_wave[w] = inc;
    __syncthreads();
    double run = s_base + (inc - local);
    for (int k = 0; k < w; ++k) run += s_wave[k];
    int hit = INT_MAX, last_pos = -1;
#pragma unroll
    for (int k = 0; k < kPerThread; ++k) {
        run += mass[k];
        if (mass[k] > 0.0) {
            last_pos = e0 + k;
            if (run > thr && hit == INT_MAX) hit = e0 + k;
        }
    }
    hit = wave_min_i(hit);
    last_pos = wave_max_i(last_pos);
    __syncthreads();
    if (lane == 0) s_i[w] = hit;
    __syncthreads();
    hit = min(min(s_i[0], s_i[1]), min(s_i[2], s_i[3]));
    __syncthreads();
    if (lane == 0) s_i[w] = last_pos;
    __syncthreads();
    last_pos = max(max(s_i[0], s_i[1]), max(s_i[2], s_i[3]));
    if (threadIdx.x == 0) {
        int tok = hit != INT_MAX ? hit : last_pos;
        if (tok < 0) tok = 0;  // unreachable for a chunk with mass; keeps the id in range
        em[dec.n] = tok;
        n_emitted[i] = dec.n + 1;
    }
}

template <int MODE, typename RT>
int launch_all(const RT* p_target, const RT* p_draft, const int32_t* draft_tokens, const float* u_accept,
               const float* u_sample, const int32_t* cu_t, const int32_t* cu_d, const int32_t* t_rows,
               const int32_t* d_rows, int32_t* accepted_len, int32_t* n_emitted, int32_t* emitted,
               const fsr_accept_params& p, const Workspace& ws_in, hipStream_t s) {
    Workspace ws = ws_in;
    const int nc = n_chunks_of(p.V);
    const double T = p.temperature;
    int rc;
#define FSR_DECIDE(PHASE)                                                                                                    \
    hipLaunchKernelGGL((accept_decide_kernel<MODE, RT, PHASE>), dim3(p.B), dim3(64), 0, s, p_target, p_draft, draft_tokens, u_accept, \
                       cu_t, cu_d, t_rows, d_rows, accepted_len, n_emitted, emitted, ws, p.B, p.V, p.S_max, T)
    if (MODE == FSR_LOGITS) {
        const int rows_cap = p.B * (2 * p.S_max + 1);
        // chunks per workgroup: as many as leave the device a few thousand workgroups (a small call is a latency
        // chain per workgroup, and more of them in parallel is what shortens it)
        int sg = kMaxStatGroup;
        while (sg > 1 && (long long)rows_cap * n_stat_groups_of(p.V, sg) < 4096) sg >>= 1;
        ws.stat_group = sg;
        const int nsg = n_stat_groups_of(p.V, sg);
    // rows of a request one pass covers: target rows T_LO .. T_LO + T_N - 1 and draft rows D_LO .. D_LO + D_N - 1
#define FSR_STATS(T_LO, T_N, D_LO, D_N, ONLY_PENDING)                                                                        \
    hipLaunchKernelGGL(accept_stats_kernel<RT>, dim3(nsg, p.B * ((T_N) + (D_N))), dim3(kThreads), 0, s, p_target, p_draft, cu_t, \
                       cu_d, t_rows, d_rows, ws, p.B, p.V, p.S_max, T, (T_N) + (D_N), T_LO, T_N, D_LO, ONLY_PENDING)
        // Only rows 0..n of a request (n = accepted drafts) have to be normalised.  With enough rows in the call to be
        // worth two more launches, the rows the first kLazyJ drafts need are normalised and those drafts tested first;
        // the remaining rows are read only for the requests that accepted all of them.
        const bool two_phase = p.S_max > kLazyJ + 1 && rows_cap >= kLazyMinRows;
        if (two_phase) {
            FSR_STATS(0, kLazyJ + 1, 0, kLazyJ, 0);
            if ((rc = check_launch("accept_stats_kernel")) != FSR_OK) return rc;
            FSR_DECIDE(1);
            if ((rc = check_launch("accept_decide_kernel")) != FSR_OK) return rc;
            FSR_STATS(kLazyJ + 1, p.S_max - kLazyJ, kLazyJ, p.S_max - kLazyJ, 1);
            if ((rc = check_launch("accept_stats_kernel")) != FSR_OK) return rc;
            FSR_DECIDE(2);
        } else {
            FSR_STATS(0, p.S_max + 1, 0, p.S_max, 0);
            if ((rc = check_launch("accept_stats_kernel")) != FSR_OK) return rc;
            FSR_DECIDE(0);
        }
#undef FSR_STATS
    } else {
        FSR_DECIDE(0);
    }
#undef FSR_DECIDE
    if ((rc = check_launch("accept_decide_kernel")) != FSR_OK) return rc;
    // chunks per workgroup: as many as leave the device about four workgroups per compute unit (a small batch
    // keeps one chunk per workgroup: there the call is a latency chain and parallelism is what shortens it)
    int group = kMaxSampleGroup;
    while (group > 1 && (long long)p.B * ((nc + group - 1) / group) < 1024) group >>= 1;
#define FSR_SAMPLE(G)                                                                                                          \
    hipLaunchKernelGGL((accept_sample_kernel<MODE, RT, G>), dim3((nc + G - 1) / G, p.B), dim3(kThreads), 0, s, p_target, p_draft, \
                       u_sample, n_emitted, emitted, ws, p.V, p.S_max, T)
    if (group == 8) FSR_SAMPLE(8);
    else if (group == 4) FSR_SAMPLE(4);
    else if (group == 2) FSR_SAMPLE(2);
    else FSR_SAMPLE(1);
#undef FSR_SAMPLE
    return check_launch("accept_sample_kernel");
}

int validate(const fsr_accept_params* p, const char* who) {
    if (!p) return fail(FSR_EINVAL, "%s: params is null", who);
    if (p->B < 0 || p->V <= 0 || p->S_max < 0 || p->reserved2 != 0)
        return fail(FSR_EINVAL, "%s: B=%d V=%d S_max=%d reserved2=%d", who, p->B, p->V, p->S_max, p->reserved2);
    if (p->dtype != FSR_F32 && p->dtype != FSR_BF16) return fail(FSR_EUNSUP, "%s: dtype=%d", who, p->dtype);
    if (p->dtype == FSR_BF16 && p->mode == FSR_GREEDY) return fail(FSR_EUNSUP, "%s: greedy mode takes fp32 rows", who);
    if (p->mode != FSR_PROBS && p->mode != FSR_LOGITS && p->mode != FSR_GREEDY) return fail(FSR_EUNSUP, "%s: mode=%d", who, p->mode);
    if (p->mode == FSR_LOGITS && !(p->temperature > 0.0)) return fail(FSR_EINVAL, "%s: temperature=%g must be > 0", who, p->temperature);
    if ((long long)p->B * (2LL * p->S_max + 1) > 65535) return fail(FSR_EUNSUP, "%s: B*(2*S_max+1)=%lld exceeds 65535 rows per call", who, (long long)p->B * (2LL * p->S_max + 1));
    return FSR_OK;
}

}  // namespace
}  // namespace fsr

using namespace fsr;

extern "C" int fsr_accept_workspace_bytes(const fsr_accept_params* p, size_t* out_bytes) {
    int rc = validate(p, "fsr_accept_workspace_bytes");
    if (rc != FSR_OK) return rc;
    if (!out_bytes) return fail(FSR_EINVAL, "fsr_accept_workspace_bytes: out_bytes is null");
    *out_bytes = p->mode == FSR_GREEDY ? greedy_workspace_bytes(*p) : carve(*p, nullptr, nullptr);
    return FSR_OK;
}

extern "C" int fsr_spec_accept(const void* p_target, const void* p_draft, const int32_t* draft_tokens,
                               const float* u_accept, const float* u_sample, const int32_t* cu_t, const int32_t* cu_d,
                               const int32_t* t_rows, const int32_t* d_rows, int32_t* accepted_len, int32_t* n_emitted,
                               int32_t* emitted, const fsr_accept_params* p, void* workspace, size_t ws_bytes,
                               void* stream) {
    int rc = validate(p, "fsr_spec_accept");
    if (rc != FSR_OK) return rc;
    if (p->B == 0) return FSR_OK;
    if (p->mode == FSR_GREEDY) {
        if (!p_target || !cu_t || !cu_d || !accepted_len || !n_emitted || !emitted)
            return fail(FSR_EINVAL, "fsr_spec_accept: null pointer among p_target/cu_t/cu_d/outputs");
        if (p->S_max > 0 && !draft_tokens) return fail(FSR_EINVAL, "fsr_spec_accept: draft_tokens is null with S_max=%d", p->S_max);
        const size_t need_g = greedy_workspace_bytes(*p);
        if (!workspace || ws_bytes < need_g) return fail(FSR_EWS, "fsr_spec_accept: workspace %zu bytes, need %zu", ws_bytes, need_g);
        if ((uintptr_t)workspace & 255) return fail(FSR_EWS, "fsr_spec_accept: workspace must be 256-byte aligned");
        return greedy_accept_launch((const float*)p_target, draft_tokens, cu_t, cu_d, t_rows, d_rows, accepted_len, n_emitted, emitted, *p,
                                    workspace, (hipStream_t)stream);
    }
    if (!p_target || !u_sample || !cu_t || !cu_d || !accepted_len || !n_emitted || !emitted)
        return fail(FSR_EINVAL, "fsr_spec_accept: null pointer among p_target/u_sample/cu_t/cu_d/outputs");
    if (p->S_max > 0 && (!p_draft || !draft_tokens || !u_accept))
        return fail(FSR_EINVAL, "fsr_spec_accept: p_draft/draft_tokens/u_accept is null with S_max=%d", p->S_max);
    Workspace ws;
    const size_t need = carve(*p, (char*)workspace, &ws);
    if (!workspace || ws_bytes < need) return fail(FSR_EWS, "fsr_spec_accept: workspace %zu bytes, need %zu", ws_bytes, need);
    if ((uintptr_t)workspace & 255) return fail(FSR_EWS, "fsr_spec_accept: workspace must be 256-byte aligned");
    hipStream_t s = (hipStream_t)stream;
    // a request without drafts never dereferences the draft arrays; give the kernels a valid base
    if (!p_draft) p_draft = p_target;
    if (p->dtype == FSR_BF16) {
        const uint16_t* pt = (const uint16_t*)p_target;
        const uint16_t* pd = (const uint16_t*)p_draft;
        if (p->mode == FSR_LOGITS)
            return launch_all<FSR_LOGITS>(pt, pd, draft_tokens, u_accept, u_sample, cu_t, cu_d, t_rows, d_rows, accepted_len,
                                          n_emitted, emitted, *p, ws, s);
        return launch_all<FSR_PROBS>(pt, pd, draft_tokens, u_accept, u_sample, cu_t, cu_d, t_rows, d_rows, accepted_len,
                                     n_emitted, emitted, *p, ws, s);
    }
    const float* pt = (const float*)p_target;
    const float* pd = (const float*)p_draft;
    if (p->mode == FSR_LOGITS)
        return launch_all<FSR_LOGITS>(pt, pd, draft_tokens, u_accept, u_sample, cu_t, cu_d, t_rows, d_rows, accepted_len,
                                      n_emitted, emitted, *p, ws, s);
    return launch_all<FSR_PROBS>(pt, pd, draft_tokens, u_accept, u_sample, cu_t, cu_d, t_rows, d_rows, accepted_len,
                                 n_emitted, emitted, *p, ws, s);
}
