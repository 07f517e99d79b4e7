// verify_attention: ragged multi-query attention of every request's draft suffix over its
// paged KV cache, causal inside the suffix (Sec. 2.1 / 3.1 of the paper: the target model
// verifies all drafted tokens of a request in one pass; every request has its own
// speculative length).
//
// Fast path (bf16, D = 128, P = 16): the op streams the KV cache once and is bound by HBM
// bandwidth, so the kernel is organised around reading K and V exactly once per KV head:
//   * one workgroup per (request, KV head, KV split); all G * q_len query rows that share
//     the KV head form the N dimension of the matrix-core tiles, so K/V bytes are reused
//     across the GQA group and across the suffix rows from registers;
//   * each of the 4 waves streams its own 32-key tiles: K goes straight from global memory
//     into the A-operand layout of v_mfma_f32_16x16x32_bf16 (S^T = K Q^T, a lane reads 64
//     contiguous bytes of one key row), V is staged through a wave-private, XOR-swizzled
//     LDS tile and read back transposed with ds_read_b64_tr_b16 (O^T = V^T P^T);
//   * S^T's accumulator layout is exactly the B-operand layout P^T needs, so the softmax
//     runs in registers with two cross-lane steps per row;
//   * P is fed to the matrix cores as a bf16 hi + lo pair: the result is accurate to fp32
//     rounding instead of bf16 rounding of the probabilities;
//   * waves, then KV splits, are merged with the usual (max, sum, weighted accumulator)
//     rule; the split merge is a second tiny kernel.
// Generic path (fp32 or bf16, D in {64,128}, any page size): one wave per (row, head), plain
// fp32 FMAs -- a correctness path for small or unusual shapes, not a bandwidth kernel.
#include "common.hpp"
#include "device_utils.hpp"

namespace fsr {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4;
typedef __attribute__((__vector_size__(8 * sizeof(short)))) short s16x8;
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

constexpr int kD = 128;           // head dim of the fast path
constexpr int kP = 16;            // page size of the fast path
constexpr int kTile = 32;         // keys per wave tile
constexpr int kWaves = 4;
constexpr int kMaxMT = 6;         // up to 96 query rows (G * rows) per pass
constexpr int kRedStride = kD + 4;  // padded row of the wave-merge buffer (floats)
// LDS: the per-wave V tiles (4 x 8 KB) and, after the key loop, the wave-merge buffer share one region
constexpr int kVTileBytes = kTile * kD * 2;
constexpr int kRedBytes = kWaves * 16 * kRedStride * 4;
constexpr int kStageBytes = kWaves * kVTileBytes > kRedBytes ? kWaves * kVTileBytes : kRedBytes;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

struct FastArgs {
    const uint16_t* q;
    const uint16_t* k;
    const uint16_t* v;
    const int32_t* bt;
    const int32_t* ctx;
    const int32_t* cu_q;
    float* part_o;   // [n_splits, N_cap, H_q, D]
    float* part_ml;  // [n_splits, N_cap, H_q, 2]  (max in log2 units, sum)
    int B, N_cap, H_q, H_kv, G, max_pages, n_pages;
    int chunk;       // keys per split (multiple of kTile * kWaves)
    int n_splits;
    float scale_log2;
};

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Swizzled byte offset of 16-byte chunk `ch` (0..15) of key row `key` in a [32][128] bf16 tile.
__device__ __forceinline__ int vtile_off(int key, int ch) { return key * 256 + ((ch ^ ((key & 7) << 1)) << 4); }

template <int MT>
__device__ void attend_rows(const FastArgs& a, int i, int kvh, int split, int c, int q0, int q_len, int j0,
                            int rows_g, char* smem) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int lg = lane >> 4, li = lane & 15;
    const int G = a.G;
    const int M_g = G * rows_g;
    const int kv_total = min(c + q_len, a.max_pages * kP);  // tokens of this request in the cache
    const int kbeg = split * a.chunk;
    const int kend = min(min(kbeg + a.chunk, c + j0 + rows_g), kv_total);  // keys any row of this pass may see
    char* vbuf = smem + w * kVTileBytes;

    // ---- Q^T operand: lane holds query row (mt*16 + li), d = 32 kk + 8 lg .. +7
    bf16x8 qreg[MT][4];
    int lim[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int m = mt * 16 + li;
        const bool ok = m < M_g;
        const int j = j0 + m / G, gq = m % G;
        lim[mt] = ok ? c + j : -1;
        const uint16_t* qp = a.q + ((size_t)(q0 + (ok ? j : j0)) * a.H_q + kvh * G + (ok ? gq : 0)) * kD + 8 * lg;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            s16x8 t = *reinterpret_cast<const s16x8*>(qp + 32 * kk);
            if (!ok) t = s16x8{0, 0, 0, 0, 0, 0, 0, 0};
            qreg[mt][kk] = __builtin_bit_cast(bf16x8, t);
        }
    }

    float m_run[MT], l_run[MT];
    f32x4 acc[MT][8];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        m_run[mt] = -INFINITY;
        l_run[mt] = 0.0f;
#pragma unroll
        for (int db = 0; db < 8; ++db) acc[mt][db] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    const int32_t* bt = a.bt + (size_t)i * a.max_pages;
    for (int kb = kbeg + w * kTile; kb < kend; kb += kWaves * kTile) {
        // ---- pages of the tile (the second page exists only if the request has tokens there)
        int pg0 = bt[kb >> 4];
        int pg1 = (kb + kP < kv_total) ? bt[(kb >> 4) + 1] : pg0;
        pg0 = min(max(pg0, 0), a.n_pages - 1);
        pg1 = min(max(pg1, 0), a.n_pages - 1);
        const uint16_t* kp0 = a.k + (((size_t)pg0 * a.H_kv + kvh) * kP + li) * kD + 8 * lg;
        const uint16_t* kp1 = a.k + (((size_t)pg1 * a.H_kv + kvh) * kP + li) * kD + 8 * lg;
        bf16x8 kreg[2][4];
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            kreg[0][kk] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const s16x8*>(kp0 + 32 * kk));
            kreg[1][kk] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const s16x8*>(kp1 + 32 * kk));
        }
        // ---- V tile: lane copies 16-byte chunk li of keys 4 r + lg, r = 0..7
        s16x8 vreg[8];
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const int key = 4 * r + lg;
            const int pg = key < kP ? pg0 : pg1;
            const uint16_t* vp = a.v + (((size_t)pg * a.H_kv + kvh) * kP + (key & 15)) * kD + 8 * li;
            vreg[r] = *reinterpret_cast<const s16x8*>(vp);
        }
        if (kb + kTile > kv_total) {  // slots past the request's last token may hold anything: zero them
#pragma unroll
            for (int r = 0; r < 8; ++r)
                if (kb + 4 * r + lg >= kv_total) vreg[r] = s16x8{0, 0, 0, 0, 0, 0, 0, 0};
        }
#pragma unroll
        for (int r = 0; r < 8; ++r) *reinterpret_cast<s16x8*>(vbuf + vtile_off(4 * r + lg, li)) = vreg[r];

        // ---- S^T = K Q^T: s[kt][e] = score(key kb + 16 kt + 4 lg + e, query mt*16 + li)
        const bool need_mask = kb + kTile > c + j0 + 1;
        bf16x8 ph[MT], pl[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            f32x4 s[2];
#pragma unroll
            for (int kt = 0; kt < 2; ++kt) {
                s[kt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int kk = 0; kk < 4; ++kk)
                    s[kt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kreg[kt][kk], qreg[mt][kk], s[kt], 0, 0, 0);
            }
            float p[8];
#pragma unroll
            for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                for (int e = 0; e < 4; ++e) p[kt * 4 + e] = s[kt][e] * a.scale_log2;
            if (need_mask) {
#pragma unroll
                for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (kb + 16 * kt + 4 * lg + e > lim[mt]) p[kt * 4 + e] = -INFINITY;
            }
            float tmax = fmaxf(fmaxf(fmaxf(p[0], p[1]), fmaxf(p[2], p[3])), fmaxf(fmaxf(p[4], p[5]), fmaxf(p[6], p[7])));
            tmax = fmaxf(tmax, __shfl_xor(tmax, 16, 64));
            tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
            const float m_new = fmaxf(m_run[mt], tmax);
            const float m_use = m_new == -INFINITY ? 0.0f : m_new;
            const float alpha = fast_exp2(m_run[mt] - m_use);
            m_run[mt] = m_new;
            float psum = 0.0f;
            // P^T as a bf16 hi + lo pair; element e < 4 is key 4 lg + e of the first 16 keys,
            // e >= 4 is key 16 + 4 lg + (e - 4): the k-order the V^T operand below uses too
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float pe = fast_exp2(p[e] - m_use);
                psum += pe;
                const __bf16 hi = (__bf16)pe;
                ph[mt][e] = hi;
                pl[mt][e] = (__bf16)(pe - (float)hi);
            }
            l_run[mt] = l_run[mt] * alpha + psum;
#pragma unroll
            for (int db = 0; db < 8; ++db) acc[mt][db] *= alpha;
        }
        // ---- O^T += V^T P^T
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
        for (int db = 0; db < 8; ++db) {
            // lane (lg, li) reads 8 bytes of key row 16 h + 4 lg + li/4 at d = 16 db + 4 (li%4);
            // after the transpose it holds keys 16 h + 4 lg + 0..3 at d = 16 db + li
            const int ch = 2 * db + ((li & 3) >> 1), half = (li & 1) * 8;
            const int r0 = 4 * lg + (li >> 2);
            const s16x4 t0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(vbuf + vtile_off(r0, ch) + half));
            const s16x4 t1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(vbuf + vtile_off(16 + r0, ch) + half));
            const s16x8 tv = s16x8{t0[0], t0[1], t0[2], t0[3], t1[0], t1[1], t1[2], t1[3]};
            const bf16x8 vop = __builtin_bit_cast(bf16x8, tv);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                acc[mt][db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vop, ph[mt], acc[mt][db], 0, 0, 0);
                acc[mt][db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vop, pl[mt], acc[mt][db], 0, 0, 0);
            }
        }
        // the next tile's V stores must not overtake this tile's transposed reads
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }

    // ---- row sums live spread over the 4 lane groups
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        l_run[mt] += __shfl_xor(l_run[mt], 16, 64);
        l_run[mt] += __shfl_xor(l_run[mt], 32, 64);
    }

    // ---- merge the 4 waves (each saw a disjoint set of keys)
    float* red_m = reinterpret_cast<float*>(smem + kStageBytes);              // [kWaves][96]
    float* red_l = red_m + kWaves * 16 * kMaxMT;
    float* red_o = reinterpret_cast<float*>(smem);                            // [kWaves][16][kRedStride], aliases vbuf
    __syncthreads();
    if (lg == 0) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            red_m[w * 16 * kMaxMT + mt * 16 + li] = m_run[mt];
            red_l[w * 16 * kMaxMT + mt * 16 + li] = l_run[mt];
        }
    }
    __syncthreads();
    const size_t prow = (size_t)split * a.N_cap;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        float m_star = -INFINITY;
#pragma unroll
        for (int ww = 0; ww < kWaves; ++ww) m_star = fmaxf(m_star, red_m[ww * 16 * kMaxMT + mt * 16 + li]);
        const float m_use = m_star == -INFINITY ? 0.0f : m_star;
        const float f = fast_exp2(m_run[mt] - m_use);
#pragma unroll
        for (int db = 0; db < 8; ++db) {
            const f32x4 o = acc[mt][db] * f;
            *reinterpret_cast<f32x4*>(red_o + (w * 16 + li) * kRedStride + db * 16 + 4 * lg) = o;
        }
        __syncthreads();
        // 256 threads sum 16 rows x 128 d over the 4 waves: thread -> row tid/16, 8 consecutive d
        {
            const int r = threadIdx.x >> 4, d0 = (threadIdx.x & 15) * 8;
            const int m = mt * 16 + r;
            f32x4 s0 = f32x4{0.f, 0.f, 0.f, 0.f}, s1 = s0;
#pragma unroll
            for (int ww = 0; ww < kWaves; ++ww) {
                s0 += *reinterpret_cast<const f32x4*>(red_o + (ww * 16 + r) * kRedStride + d0);
                s1 += *reinterpret_cast<const f32x4*>(red_o + (ww * 16 + r) * kRedStride + d0 + 4);
            }
            if (m < M_g) {
                const int j = j0 + m / G, h = kvh * G + m % G;
                float* dst = a.part_o + ((prow + q0 + j) * a.H_q + h) * kD + d0;
                *reinterpret_cast<f32x4*>(dst) = s0;
                *reinterpret_cast<f32x4*>(dst + 4) = s1;
                if ((threadIdx.x & 15) == 0) {
                    float ms = -INFINITY;
#pragma unroll
                    for (int ww = 0; ww < kWaves; ++ww) ms = fmaxf(ms, red_m[ww * 16 * kMaxMT + m]);
                    const float mu = ms == -INFINITY ? 0.0f : ms;
                    float ls = 0.0f;
#pragma unroll
                    for (int ww = 0; ww < kWaves; ++ww)
                        ls += red_l[ww * 16 * kMaxMT + m] * fast_exp2(red_m[ww * 16 * kMaxMT + m] - mu);
                    float* ml = a.part_ml + ((prow + q0 + j) * a.H_q + h) * 2;
                    ml[0] = ms;
                    ml[1] = ls;
                }
            }
        }
        __syncthreads();
    }
}

constexpr int kFastSmem = kStageBytes + 2 * kWaves * 16 * kMaxMT * 4;

// grid = (n_splits, H_kv, B), block = 256.  MTMAX bounds the 16-row query tiles a pass may hold
// (and with it the register budget); requests with more rows take several passes over their keys.
template <int MTMAX>
__global__ __launch_bounds__(256) void attn_fast_kernel(FastArgs a) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int split = blockIdx.x, kvh = blockIdx.y, i = blockIdx.z;
    const int q0 = a.cu_q[i], q_len = a.cu_q[i + 1] - q0;
    if (q_len <= 0) return;
    const int c = a.ctx[i];
    if (split * a.chunk >= c + q_len) return;  // this split holds no key of the request
    const int rows_per_pass = (16 * MTMAX) / a.G;
    for (int j0 = 0; j0 < q_len; j0 += rows_per_pass) {
        const int rows_g = min(rows_per_pass, q_len - j0);
        const int mt = (a.G * rows_g + 15) >> 4;
        if constexpr (MTMAX == 1) {
            attend_rows<1>(a, i, kvh, split, c, q0, q_len, j0, rows_g, smem);
        } else if constexpr (MTMAX == 2) {
            if (mt == 1) attend_rows<1>(a, i, kvh, split, c, q0, q_len, j0, rows_g, smem);
            else attend_rows<2>(a, i, kvh, split, c, q0, q_len, j0, rows_g, smem);
        } else if constexpr (MTMAX == 3) {
            if (mt == 1) attend_rows<1>(a, i, kvh, split, c, q0, q_len, j0, rows_g, smem);
            else if (mt == 2) attend_rows<2>(a, i, kvh, split, c, q0, q_len, j0, rows_g, smem);
            else attend_rows<3>(a, i, kvh, split, c, q0, q_len, j0, rows_g, smem);
        } else if constexpr (MTMAX == 4) {
            if (mt <= 2) attend_rows<2>(a, i, kvh, split, c, q0, q_len, j0, rows_g, smem);
            else if (mt == 3) attend_rows<3>(a, i, kvh, split, c, q0, q_len, j0, rows_g, smem);
            else attend_rows<4>(a, i, kvh, split, c, q0, q_len, j0, rows_g, smem);
        } else {
            if (mt <= 2) attend_rows<2>(a, i, kvh, split, c, q0, q_len, j0, rows_g, smem);
            else if (mt <= 4) attend_rows<4>(a, i, kvh, split, c, q0, q_len, j0, rows_g, smem);
            else attend_rows<6>(a, i, kvh, split, c, q0, q_len, j0, rows_g, smem);
        }
        __syncthreads();
    }
}

__device__ __forceinline__ int find_request(const int32_t* __restrict__ cu_q, int B, int row) {
    int lo = 0, hi = B;  // largest i with cu_q[i] <= row, skipping empty requests to the right
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (cu_q[mid] <= row) lo = mid; else hi = mid;
    }
    return lo;
}

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float x) { return __builtin_bit_cast(uint16_t, (__bf16)x); }

// Merge the KV splits of one row.  grid = (N_cap), block = 256 (thread -> 4 consecutive d of one head per step)
template <typename OutT>
__global__ __launch_bounds__(256) void attn_merge_kernel(FastArgs a, OutT* __restrict__ out, float* __restrict__ lse) {
    const int row = blockIdx.x;
    if (row >= a.cu_q[a.B]) return;
    const int i = find_request(a.cu_q, a.B, row);
    const int kv_total = a.ctx[i] + (a.cu_q[i + 1] - a.cu_q[i]);
    const int ns = min((kv_total + a.chunk - 1) / a.chunk, a.n_splits);
    const size_t stride_o = (size_t)a.N_cap * a.H_q * kD, stride_ml = (size_t)a.N_cap * a.H_q * 2;
    for (int e = threadIdx.x; e < a.H_q * (kD / 4); e += blockDim.x) {
        const int h = e / (kD / 4), d0 = (e % (kD / 4)) * 4;
        const float* ml = a.part_ml + ((size_t)row * a.H_q + h) * 2;
        float m_star = -INFINITY;
        for (int s = 0; s < ns; ++s) m_star = fmaxf(m_star, ml[s * stride_ml]);
        const float mu = m_star == -INFINITY ? 0.0f : m_star;
        f32x4 o = f32x4{0.f, 0.f, 0.f, 0.f};
        float l = 0.0f;
        const float* po = a.part_o + ((size_t)row * a.H_q + h) * kD + d0;
        for (int s = 0; s < ns; ++s) {
            const float wgt = fast_exp2(ml[s * stride_ml] - mu);
            l += ml[s * stride_ml + 1] * wgt;
            o += *reinterpret_cast<const f32x4*>(po + s * stride_o) * wgt;
        }
        const float inv = 1.0f / l;
        OutT* dst = out + ((size_t)row * a.H_q + h) * kD + d0;
        if constexpr (sizeof(OutT) == 4) {
            *reinterpret_cast<f32x4*>(dst) = o * inv;
        } else {
            ushort4 pk;
            pk.x = f32_to_bf16_rne(o[0] * inv);
            pk.y = f32_to_bf16_rne(o[1] * inv);
            pk.z = f32_to_bf16_rne(o[2] * inv);
            pk.w = f32_to_bf16_rne(o[3] * inv);
            *reinterpret_cast<ushort4*>(dst) = pk;
        }
        if (lse && d0 == 0) lse[(size_t)row * a.H_q + h] = (m_star + __log2f(l)) * kLn2;
    }
}

// ---------------------------------------------------------------------------------------
// Generic path: one wave per (row, head); lanes stride over the keys.
// ---------------------------------------------------------------------------------------
struct GenericArgs {
    const void* q;
    const void* k;
    const void* v;
    const int32_t* bt;
    const int32_t* ctx;
    const int32_t* cu_q;
    void* out;
    float* lse;
    int B, H_q, H_kv, P, max_pages, n_pages;
    float scale;
};

template <typename T>
__device__ __forceinline__ float to_f32(T x);
template <>
__device__ __forceinline__ float to_f32<float>(float x) { return x; }
template <>
__device__ __forceinline__ float to_f32<uint16_t>(uint16_t x) { return __builtin_bit_cast(float, (uint32_t)x << 16); }

template <typename T, typename OutT, int D>
__global__ __launch_bounds__(64) void attn_generic_kernel(GenericArgs a) {
    __shared__ float qs[D];
    const int h = blockIdx.x, row = blockIdx.y, lane = threadIdx.x;
    if (row >= a.cu_q[a.B]) return;
    const int i = find_request(a.cu_q, a.B, row);
    const int j = row - a.cu_q[i];
    const int L = min(a.ctx[i] + j + 1, a.max_pages * a.P);
    const int g = h / (a.H_q / a.H_kv);
    const T* q = reinterpret_cast<const T*>(a.q) + ((size_t)row * a.H_q + h) * D;
    for (int d = lane; d < D; d += 64) qs[d] = to_f32<T>(q[d]);
    __syncthreads();
    float m = -INFINITY, l = 0.0f;
    float o[D];
#pragma unroll
    for (int d = 0; d < D; ++d) o[d] = 0.0f;
    const int32_t* bt = a.bt + (size_t)i * a.max_pages;
    const T* kc = reinterpret_cast<const T*>(a.k);
    const T* vc = reinterpret_cast<const T*>(a.v);
    for (int t = lane; t < L; t += 64) {
        const int pg = min(max(bt[t / a.P], 0), a.n_pages - 1);
        const size_t base = (((size_t)pg * a.H_kv + g) * a.P + t % a.P) * D;
        float s = 0.0f;
#pragma unroll
        for (int d = 0; d < D; ++d) s = fmaf(qs[d], to_f32<T>(kc[base + d]), s);
        s *= a.scale;
        const float m_new = fmaxf(m, s);
        const float alpha = expf(m - m_new), p = expf(s - m_new);
        l = l * alpha + p;
#pragma unroll
        for (int d = 0; d < D; ++d) o[d] = fmaf(p, to_f32<T>(vc[base + d]), o[d] * alpha);
        m = m_new;
    }
    const float m_star = wave_max(m);  // L >= 1: lane 0 always has a key
    const float f = m == -INFINITY ? 0.0f : expf(m - m_star);
    float ls = l * f;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) ls += __shfl_xor(ls, off, 64);
    const float inv = 1.0f / ls;
    OutT* out = reinterpret_cast<OutT*>(a.out) + ((size_t)row * a.H_q + h) * D;
#pragma unroll
    for (int d = 0; d < D; ++d) {
        float x = o[d] * f;
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off, 64);
        if (lane == (d & 63)) {
            if constexpr (sizeof(OutT) == 4) out[d] = x * inv;
            else out[d] = f32_to_bf16_rne(x * inv);
        }
    }
    if (a.lse && lane == 0) a.lse[(size_t)row * a.H_q + h] = m_star + logf(ls);
}

struct Plan {
    bool fast;
    int mt_max;  // 16-row query tiles per pass of the fast kernel
    int chunk, n_splits;
    size_t bytes_o, bytes_ml;
};

int validate(const fsr_attn_params* p, const char* who) {
    if (!p) return fail(FSR_EINVAL, "%s: params is null", who);
    if (p->max_q_len < 0) return fail(FSR_EINVAL, "%s: max_q_len=%d", who, p->max_q_len);
    if (p->B < 0 || p->N_cap < 0 || p->H_q <= 0 || p->H_kv <= 0 || p->max_pages <= 0 || p->n_pages <= 0 || p->P <= 0 || p->reserved != 0)
        return fail(FSR_EINVAL, "%s: B=%d N_cap=%d H_q=%d H_kv=%d max_pages=%d n_pages=%d P=%d reserved=%d", who, p->B, p->N_cap,
                    p->H_q, p->H_kv, p->max_pages, p->n_pages, p->P, p->reserved);
    if (p->H_q % p->H_kv != 0) return fail(FSR_ESHAPE, "%s: H_q=%d is not a multiple of H_kv=%d", who, p->H_q, p->H_kv);
    if (p->D != 64 && p->D != 128) return fail(FSR_EUNSUP, "%s: head dim %d (64 and 128 are built)", who, p->D);
    if (p->dtype != FSR_F32 && p->dtype != FSR_BF16) return fail(FSR_EUNSUP, "%s: dtype=%d", who, p->dtype);
    if (p->out_dtype != FSR_F32 && !(p->out_dtype == FSR_BF16 && p->dtype == FSR_BF16))
        return fail(FSR_EUNSUP, "%s: out_dtype=%d with dtype=%d", who, p->out_dtype, p->dtype);
    if (!(p->scale > 0.0f)) return fail(FSR_EINVAL, "%s: scale=%g must be > 0", who, (double)p->scale);
    if (p->B > 65535 || p->H_kv > 65535) return fail(FSR_EUNSUP, "%s: B and H_kv are limited to 65535", who);
    return FSR_OK;
}

Plan make_plan(const fsr_attn_params& p) {
    Plan pl{};
    const int G = p.H_q / p.H_kv;
    pl.fast = p.dtype == FSR_BF16 && p.D == kD && p.P == kP && G <= 16 && (16 * kMaxMT) / G >= 1;
    if (!pl.fast) return pl;
    // rows of one request that share a KV head: G * max_q_len (unknown bound -> the widest kernel)
    const long long m_rows = p.max_q_len > 0 ? (long long)G * p.max_q_len : 16 * kMaxMT;
    const int mt = (int)std::min<long long>((m_rows + 15) / 16, kMaxMT);
    pl.mt_max = mt <= 4 ? mt : kMaxMT;
    // Over-decompose the KV axis so that the batch fills 256 CUs several times over even when
    // it has few (request, KV head) pairs; the lengths live on the device, so the grid covers
    // the capacity max_pages * P and splits beyond a request's length exit at once.
    const long long cap = (long long)p.max_pages * kP;
    const long long items = std::max(1LL, (long long)p.B * p.H_kv);
    const long long want = std::max(1LL, (2048 + items - 1) / items);
    const int unit = kTile * kWaves;
    long long chunk = (cap + want - 1) / want;
    chunk = std::max<long long>(2 * unit, (chunk + unit - 1) / unit * unit);
    pl.chunk = (int)chunk;
    pl.n_splits = (int)((cap + chunk - 1) / chunk);
    pl.bytes_o = align_up((size_t)pl.n_splits * p.N_cap * p.H_q * kD * sizeof(float), 256);
    pl.bytes_ml = align_up((size_t)pl.n_splits * p.N_cap * p.H_q * 2 * sizeof(float), 256);
    return pl;
}

}  // namespace
}  // namespace fsr

using namespace fsr;

extern "C" int fsr_attn_workspace_bytes(const fsr_attn_params* p, size_t* out_bytes) {
    int rc = validate(p, "fsr_attn_workspace_bytes");
    if (rc != FSR_OK) return rc;
    if (!out_bytes) return fail(FSR_EINVAL, "fsr_attn_workspace_bytes: out_bytes is null");
    const Plan pl = make_plan(*p);
    *out_bytes = pl.fast ? pl.bytes_o + pl.bytes_ml : 0;
    return FSR_OK;
}

extern "C" int fsr_verify_attention(const void* q, const void* k_cache, const void* v_cache,
                                    const int32_t* block_tables, const int32_t* ctx_lens, const int32_t* spec_lens,
                                    const int32_t* cu_q, void* out, float* lse, const fsr_attn_params* p,
                                    void* workspace, size_t ws_bytes, void* stream) {
    (void)spec_lens;
    int rc = validate(p, "fsr_verify_attention");
    if (rc != FSR_OK) return rc;
    if (p->B == 0 || p->N_cap == 0) return FSR_OK;
    if (!q || !k_cache || !v_cache || !block_tables || !ctx_lens || !cu_q || !out)
        return fail(FSR_EINVAL, "fsr_verify_attention: null pointer among q/k_cache/v_cache/block_tables/ctx_lens/cu_q/out");
    if (p->N_cap > 65535 * 32) return fail(FSR_EUNSUP, "fsr_verify_attention: N_cap=%d too large", p->N_cap);
    hipStream_t s = (hipStream_t)stream;
    const Plan pl = make_plan(*p);
    if (pl.fast) {
        const size_t need = pl.bytes_o + pl.bytes_ml;
        if (!workspace || ws_bytes < need) return fail(FSR_EWS, "fsr_verify_attention: workspace %zu bytes, need %zu", ws_bytes, need);
        if ((uintptr_t)workspace & 255) return fail(FSR_EWS, "fsr_verify_attention: workspace must be 256-byte aligned");
        if (((uintptr_t)q | (uintptr_t)k_cache | (uintptr_t)v_cache | (uintptr_t)out) & 15)
            return fail(FSR_EINVAL, "fsr_verify_attention: q/k_cache/v_cache/out must be 16-byte aligned");
        FastArgs a;
        a.q = (const uint16_t*)q; a.k = (const uint16_t*)k_cache; a.v = (const uint16_t*)v_cache;
        a.bt = block_tables; a.ctx = ctx_lens; a.cu_q = cu_q;
        a.part_o = (float*)workspace;
        a.part_ml = (float*)((char*)workspace + pl.bytes_o);
        a.B = p->B; a.N_cap = p->N_cap; a.H_q = p->H_q; a.H_kv = p->H_kv; a.G = p->H_q / p->H_kv;
        a.max_pages = p->max_pages; a.n_pages = p->n_pages; a.chunk = pl.chunk; a.n_splits = pl.n_splits;
        a.scale_log2 = p->scale * kLog2e;
        const dim3 grid(pl.n_splits, p->H_kv, p->B), block(256);
        switch (pl.mt_max) {
            case 1: hipLaunchKernelGGL(attn_fast_kernel<1>, grid, block, kFastSmem, s, a); break;
            case 2: hipLaunchKernelGGL(attn_fast_kernel<2>, grid, block, kFastSmem, s, a); break;
            case 3: hipLaunchKernelGGL(attn_fast_kernel<3>, grid, block, kFastSmem, s, a); break;
            case 4: hipLaunchKernelGGL(attn_fast_kernel<4>, grid, block, kFastSmem, s, a); break;
            default: hipLaunchKernelGGL(attn_fast_kernel<6>, grid, block, kFastSmem, s, a); break;
        }
        if ((rc = check_launch("attn_fast_kernel")) != FSR_OK) return rc;
        if (p->out_dtype == FSR_BF16)
            hipLaunchKernelGGL(attn_merge_kernel<uint16_t>, dim3(p->N_cap), dim3(256), 0, s, a, (uint16_t*)out, lse);
        else
            hipLaunchKernelGGL(attn_merge_kernel<float>, dim3(p->N_cap), dim3(256), 0, s, a, (float*)out, lse);
        return check_launch("attn_merge_kernel");
    }
    GenericArgs g;
    g.q = q; g.k = k_cache; g.v = v_cache; g.bt = block_tables; g.ctx = ctx_lens; g.cu_q = cu_q; g.out = out; g.lse = lse;
    g.B = p->B; g.H_q = p->H_q; g.H_kv = p->H_kv; g.P = p->P; g.max_pages = p->max_pages; g.n_pages = p->n_pages;
    g.scale = p->scale;
    const dim3 grid(p->H_q, p->N_cap), block(64);
    if (p->N_cap > 65535) return fail(FSR_EUNSUP, "fsr_verify_attention: generic path is limited to N_cap <= 65535 rows");
    const bool bf_in = p->dtype == FSR_BF16, bf_out = p->out_dtype == FSR_BF16;
    if (p->D == 64) {
        if (!bf_in) hipLaunchKernelGGL((attn_generic_kernel<float, float, 64>), grid, block, 0, s, g);
        else if (bf_out) hipLaunchKernelGGL((attn_generic_kernel<uint16_t, uint16_t, 64>), grid, block, 0, s, g);
        else hipLaunchKernelGGL((attn_generic_kernel<uint16_t, float, 64>), grid, block, 0, s, g);
    } else {
        if (!bf_in) hipLaunchKernelGGL((attn_generic_kernel<float, float, 128>), grid, block, 0, s, g);
        else if (bf_out) hipLaunchKernelGGL((attn_generic_kernel<uint16_t, uint16_t, 128>), grid, block, 0, s, g);
        else hipLaunchKernelGGL((attn_generic_kernel<uint16_t, float, 128>), grid, block, 0, s, g);
    }
    return check_launch("attn_generic_kernel");
}
