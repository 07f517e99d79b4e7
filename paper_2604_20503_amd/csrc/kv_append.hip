// Cache append (Sec. 2.1 / Sec. 3.1: the drafted tokens of a request enter the target model as new
// positions behind its cached context): the keys and values of a call's rows are stored into the
// request's pages before the attention of the same forward pass reads them.
//
// Pure data movement, a few hundred KB per call: one thread moves 16 bytes of one (row, KV head)
// vector of K and of V; consecutive threads cover a vector, so loads and stores are coalesced over
// D * elem bytes (256 bytes for bf16, D = 128).
#include <cstdint>

#include "common.hpp"

namespace fsr {
namespace {

constexpr int kThreads = 256;

typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;

struct AppendArgs {
    const char* k_new;
    const char* v_new;
    char* k_cache;
    char* v_cache;
    const int32_t* bt;
    const int32_t* ctx;
    const int32_t* cu_q;
    int B, N_cap, H_kv, P, max_pages, n_pages;
    int token_major;  // 1: caches are [page][P][H_kv][D], 0: [page][H_kv][P][D]
    int vec_bytes;  // D * element size, a multiple of 16
};

__device__ __forceinline__ int owner(const int32_t* __restrict__ cu, int B, int x) {
    int lo = 0, hi = B;  // largest i with cu[i] <= x, skipping empty requests to the right
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (cu[mid] <= x) lo = mid; else hi = mid;
    }
    return lo;
}

__global__ __launch_bounds__(kThreads) void kv_append_kernel(AppendArgs a) {
    const int per_vec = a.vec_bytes / 16;                       // 16-byte pieces of one (row, head) vector
    const long long piece = (long long)blockIdx.x * kThreads + threadIdx.x;
    const long long vec_id = piece / per_vec;                   // (row, head)
    const int part = (int)(piece % per_vec);
    const int row = (int)(vec_id / a.H_kv), g = (int)(vec_id % a.H_kv);
    if (row >= a.N_cap || row >= a.cu_q[a.B]) return;
    const int i = owner(a.cu_q, a.B, row);
    const long long t = (long long)a.ctx[i] + (row - a.cu_q[i]);
    if (t < 0 || t >= (long long)a.max_pages * a.P) return;     // no page for this position
    const int page = a.bt[(size_t)i * a.max_pages + t / a.P];
    if (page < 0 || page >= a.n_pages) return;                  // never write outside the pool
    const size_t src = ((size_t)row * a.H_kv + g) * a.vec_bytes + (size_t)part * 16;
    const size_t slot = a.token_major ? ((size_t)page * a.P + t % a.P) * a.H_kv + g : ((size_t)page * a.H_kv + g) * a.P + t % a.P;
    const size_t dst = slot * a.vec_bytes + (size_t)part * 16;
    *reinterpret_cast<u32x4*>(a.k_cache + dst) = *reinterpret_cast<const u32x4*>(a.k_new + src);
    *reinterpret_cast<u32x4*>(a.v_cache + dst) = *reinterpret_cast<const u32x4*>(a.v_new + src);
}

// The same append into 8-bit caches: one thread takes 16 bf16 elements of one (row, KV head) vector of K and of
// V, divides by the head's scale in fp32, rounds to E4M3 (nearest even; beyond +-448 the largest finite value;
// NaN stays NaN) and stores 16 bytes.
struct Append8Args {
    const uint16_t* k_new;
    const uint16_t* v_new;
    uint8_t* k_cache;
    uint8_t* v_cache;
    const float* k_scale;
    const float* v_scale;
    const int32_t* bt;
    const int32_t* ctx;
    const int32_t* cu_q;
    int B, N_cap, H_kv, D, P, max_pages, n_pages;
    int token_major;
};

__device__ __forceinline__ float bf16_bits_to_float(uint32_t h) { return __builtin_bit_cast(float, h << 16); }

// Two fp32 values -> two E4M3 bytes in the low or high half of `old`.
__device__ __forceinline__ uint32_t pack_e4m3(float x, float y, uint32_t old, bool high) {
    // the conversion instruction rounds to nearest even; saturation and NaN are made explicit here
    const float cx = fminf(fmaxf(x, -448.0f), 448.0f), cy = fminf(fmaxf(y, -448.0f), 448.0f);
    uint32_t w = high ? (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(cx, cy, (int)old, true)
                      : (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(cx, cy, (int)old, false);
    const int sh = high ? 16 : 0;
    if (x != x) w = (w & ~(0xffu << sh)) | (0x7fu << sh);
    if (y != y) w = (w & ~(0xffu << (sh + 8))) | (0x7fu << (sh + 8));
    return w;
}

__device__ __forceinline__ u32x4 quantise16(const uint16_t* src, float scale) {
    // (elements to scalars before use: see rank_check.hip on bit casts of vector-element expressions)
    const u32x4 lo = *reinterpret_cast<const u32x4*>(src), hi = *reinterpret_cast<const u32x4*>(src + 8);
    const uint32_t in[8] = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    uint32_t out[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const uint32_t a = in[2 * k], b = in[2 * k + 1];  // four consecutive elements
        const float x0 = bf16_bits_to_float(a & 0xffffu) / scale, x1 = bf16_bits_to_float(a >> 16) / scale;
        const float x2 = bf16_bits_to_float(b & 0xffffu) / scale, x3 = bf16_bits_to_float(b >> 16) / scale;
        out[k] = pack_e4m3(x2, x3, pack_e4m3(x0, x1, 0u, false), true);
    }
    return u32x4{out[0], out[1], out[2], out[3]};
}

__global__ __launch_bounds__(kThreads) void kv_append8_kernel(Append8Args a) {
    const int per_vec = a.D / 16;                               // 16-element pieces of one (row, head) vector
    const long long piece = (long long)blockIdx.x * kThreads + threadIdx.x;
    const long long vec_id = piece / per_vec;
    const int part = (int)(piece % per_vec);
    const int row = (int)(vec_id / a.H_kv), g = (int)(vec_id % a.H_kv);
    if (row >= a.N_cap || row >= a.cu_q[a.B]) return;
    const int i = owner(a.cu_q, a.B, row);
    const long long t = (long long)a.ctx[i] + (row - a.cu_q[i]);
    if (t < 0 || t >= (long long)a.max_pages * a.P) return;     // no page for this position
    const int page = a.bt[(size_t)i * a.max_pages + t / a.P];
    if (page < 0 || page >= a.n_pages) return;                  // never write outside the pool
    const size_t src = ((size_t)row * a.H_kv + g) * a.D + (size_t)part * 16;
    const size_t slot = a.token_major ? ((size_t)page * a.P + t % a.P) * a.H_kv + g : ((size_t)page * a.H_kv + g) * a.P + t % a.P;
    const size_t dst = slot * a.D + (size_t)part * 16;
    *reinterpret_cast<u32x4*>(a.k_cache + dst) = quantise16(a.k_new + src, a.k_scale[g]);
    *reinterpret_cast<u32x4*>(a.v_cache + dst) = quantise16(a.v_new + src, a.v_scale[g]);
}

}  // namespace
}  // namespace fsr

using namespace fsr;

extern "C" int fsr_kv_append_kv8(const void* k_new, const void* v_new, void* k_cache, void* v_cache, const float* k_scale,
                                 const float* v_scale, const int32_t* block_tables, const int32_t* ctx_lens,
                                 const int32_t* cu_q, const fsr_attn_params* p, void* stream) {
    if (!p) return fail(FSR_EINVAL, "fsr_kv_append_kv8: params is null");
    if (p->B < 0 || p->N_cap < 0 || p->H_kv <= 0 || p->D <= 0 || p->P <= 0 || p->max_pages <= 0 || p->n_pages <= 0)
        return fail(FSR_EINVAL, "fsr_kv_append_kv8: B=%d N_cap=%d H_kv=%d D=%d P=%d max_pages=%d n_pages=%d", p->B, p->N_cap,
                    p->H_kv, p->D, p->P, p->max_pages, p->n_pages);
    if (p->dtype != FSR_BF16) return fail(FSR_EUNSUP, "fsr_kv_append_kv8: rows must be bf16 (dtype=%d)", p->dtype);
    if (p->kv_layout != FSR_KV_HEAD_MAJOR && p->kv_layout != FSR_KV_TOKEN_MAJOR) return fail(FSR_EINVAL, "fsr_kv_append_kv8: kv_layout=%d", p->kv_layout);
    if (p->D % 16 != 0) return fail(FSR_EUNSUP, "fsr_kv_append_kv8: D=%d, need a multiple of 16", p->D);
    if (p->B == 0 || p->N_cap == 0) return FSR_OK;
    if (!k_new || !v_new || !k_cache || !v_cache || !k_scale || !v_scale || !block_tables || !ctx_lens || !cu_q)
        return fail(FSR_EINVAL, "fsr_kv_append_kv8: null pointer among k_new/v_new/k_cache/v_cache/k_scale/v_scale/block_tables/ctx_lens/cu_q");
    if (((uintptr_t)k_new | (uintptr_t)v_new | (uintptr_t)k_cache | (uintptr_t)v_cache) & 15)
        return fail(FSR_EINVAL, "fsr_kv_append_kv8: k_new/v_new/k_cache/v_cache must be 16-byte aligned");
    Append8Args a;
    a.k_new = (const uint16_t*)k_new; a.v_new = (const uint16_t*)v_new; a.k_cache = (uint8_t*)k_cache; a.v_cache = (uint8_t*)v_cache;
    a.k_scale = k_scale; a.v_scale = v_scale;
    a.bt = block_tables; a.ctx = ctx_lens; a.cu_q = cu_q;
    a.B = p->B; a.N_cap = p->N_cap; a.H_kv = p->H_kv; a.D = p->D; a.P = p->P; a.max_pages = p->max_pages; a.n_pages = p->n_pages;
    a.token_major = p->kv_layout == FSR_KV_TOKEN_MAJOR;
    const long long pieces = (long long)p->N_cap * p->H_kv * (p->D / 16);
    const long long blocks = (pieces + kThreads - 1) / kThreads;
    if (blocks > 0x7fffffffLL) return fail(FSR_EUNSUP, "fsr_kv_append_kv8: N_cap * H_kv * D too large for one launch");
    hipLaunchKernelGGL(kv_append8_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, (hipStream_t)stream, a);
    return check_launch("kv_append8_kernel");
}

extern "C" int fsr_kv_append(const void* k_new, const void* v_new, void* k_cache, void* v_cache,
                             const int32_t* block_tables, const int32_t* ctx_lens, const int32_t* cu_q,
                             const fsr_attn_params* p, void* stream) {
    if (!p) return fail(FSR_EINVAL, "fsr_kv_append: params is null");
    if (p->B < 0 || p->N_cap < 0 || p->H_kv <= 0 || p->D <= 0 || p->P <= 0 || p->max_pages <= 0 || p->n_pages <= 0)
        return fail(FSR_EINVAL, "fsr_kv_append: B=%d N_cap=%d H_kv=%d D=%d P=%d max_pages=%d n_pages=%d", p->B, p->N_cap,
                    p->H_kv, p->D, p->P, p->max_pages, p->n_pages);
    if (p->dtype != FSR_F32 && p->dtype != FSR_BF16) return fail(FSR_EUNSUP, "fsr_kv_append: dtype=%d", p->dtype);
    if (p->kv_layout != FSR_KV_HEAD_MAJOR && p->kv_layout != FSR_KV_TOKEN_MAJOR) return fail(FSR_EINVAL, "fsr_kv_append: kv_layout=%d", p->kv_layout);
    const int vec_bytes = p->D * (p->dtype == FSR_F32 ? 4 : 2);
    if (vec_bytes % 16 != 0) return fail(FSR_EUNSUP, "fsr_kv_append: D=%d gives %d-byte vectors, need a multiple of 16", p->D, vec_bytes);
    if (p->B == 0 || p->N_cap == 0) return FSR_OK;
    if (!k_new || !v_new || !k_cache || !v_cache || !block_tables || !ctx_lens || !cu_q)
        return fail(FSR_EINVAL, "fsr_kv_append: null pointer among k_new/v_new/k_cache/v_cache/block_tables/ctx_lens/cu_q");
    if (((uintptr_t)k_new | (uintptr_t)v_new | (uintptr_t)k_cache | (uintptr_t)v_cache) & 15)
        return fail(FSR_EINVAL, "fsr_kv_append: k_new/v_new/k_cache/v_cache must be 16-byte aligned");
    AppendArgs a;
    a.k_new = (const char*)k_new; a.v_new = (const char*)v_new; a.k_cache = (char*)k_cache; a.v_cache = (char*)v_cache;
    a.bt = block_tables; a.ctx = ctx_lens; a.cu_q = cu_q;
    a.B = p->B; a.N_cap = p->N_cap; a.H_kv = p->H_kv; a.P = p->P; a.max_pages = p->max_pages; a.n_pages = p->n_pages;
    a.vec_bytes = vec_bytes;
    a.token_major = p->kv_layout == FSR_KV_TOKEN_MAJOR;
    const long long pieces = (long long)p->N_cap * p->H_kv * (vec_bytes / 16);
    const long long blocks = (pieces + kThreads - 1) / kThreads;
    if (blocks > 0x7fffffffLL) return fail(FSR_EUNSUP, "fsr_kv_append: N_cap * H_kv * D too large for one launch");
    hipLaunchKernelGGL(kv_append_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, (hipStream_t)stream, a);
    return check_launch("kv_append_kernel");
}
