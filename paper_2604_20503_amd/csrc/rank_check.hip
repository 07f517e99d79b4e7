// Early-exit rank check (Sec. 3.2: intermediate scores predict a rejection when the draft is not
// among their K best tokens; Sec. 4: decided by counting the scores above the draft's own, without
// building the set of the K best).
//
// The work is one pass over the score row of every draft that still has an active row: count the
// scores strictly above the draft's own.  That is HBM streaming with a trivial reduction, so the
// kernels are laid out for bandwidth: a grid of (32 KB chunk of a row) x (draft), 16-byte loads,
// one integer atomic per workgroup into the draft's rank.
//
//   rank_init_kernel    rank[d] = 0 for drafts with an active row and a valid token id, -1 for
//                       drafts without a row, V for ids outside the vocabulary
//   rank_count_kernel   rank[d] += #{v in chunk : z[row][v] > z[row][draft]}
//   rank_mask_kernel    keep[row] from the ranks (first row of a request always kept)
#include <cstdint>

#include "common.hpp"
#include "device_utils.hpp"

namespace fsr {
namespace {

constexpr int kThreads = 256;
constexpr int kChunk = 8192;  // scores per workgroup: 32 KB of fp32, 16 KB of bf16

typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;

struct RankArgs {
    const void* logits;
    const int32_t* draft_tokens;
    const int32_t* cu_q;
    const int32_t* cu_d;
    int32_t* rank;
    uint8_t* keep;
    int B, V, K, N_cap, D_cap;
};

// Largest i with cu[i] <= x, skipping empty requests to the right (cu is non-decreasing, cu[0] = 0).
__device__ __forceinline__ int owner(const int32_t* __restrict__ cu, int B, int x) {
    int lo = 0, hi = B;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (cu[mid] <= x) lo = mid; else hi = mid;
    }
    return lo;
}

// Score row of draft d, or -1 if the draft has no active row (its rows were pruned earlier).
__device__ __forceinline__ int row_of_draft(const RankArgs& a, int d) {
    const int i = owner(a.cu_d, a.B, d);
    const int j = d - a.cu_d[i];
    return j < a.cu_q[i + 1] - a.cu_q[i] ? a.cu_q[i] + j : -1;
}

template <typename T>
__device__ __forceinline__ float score(const void* base, size_t idx);
template <>
__device__ __forceinline__ float score<float>(const void* base, size_t idx) {
    return reinterpret_cast<const float*>(base)[idx];
}
template <>
__device__ __forceinline__ float score<uint16_t>(const void* base, size_t idx) {
    return __builtin_bit_cast(float, (uint32_t)reinterpret_cast<const uint16_t*>(base)[idx] << 16);
}

// How many of the two bf16 scores packed in w exceed x.
__device__ __forceinline__ int above_pair(uint32_t w, float x) {
    return (__builtin_bit_cast(float, w << 16) > x) + (__builtin_bit_cast(float, w & 0xffff0000u) > x);
}

__global__ __launch_bounds__(kThreads) void rank_init_kernel(RankArgs a) {
    const int d = blockIdx.x * kThreads + threadIdx.x;
    if (d >= a.D_cap || d >= a.cu_d[a.B]) return;
    const int row = row_of_draft(a, d);
    const int tok = a.draft_tokens[d];
    a.rank[d] = row < 0 ? -1 : (tok < 0 || tok >= a.V) ? a.V : 0;
}

template <typename T>
__global__ __launch_bounds__(kThreads) void rank_count_kernel(RankArgs a) {
    __shared__ int part[kThreads / 64];
    const int d = blockIdx.y;
    if (d >= a.cu_d[a.B]) return;
    const int row = row_of_draft(a, d);
    const int tok = a.draft_tokens[d];
    if (row < 0 || row >= a.N_cap || tok < 0 || tok >= a.V) return;  // uniform for the workgroup
    const size_t base = (size_t)row * a.V;
    const float mine = score<T>(a.logits, base + tok);
    const int v0 = blockIdx.x * kChunk, v1 = min(v0 + kChunk, a.V);
    constexpr int kPer = 16 / sizeof(T);  // scores per 16-byte load
    int count = 0;
    // a row starts at any element offset: peel up to the first 16-byte boundary of the chunk
    const uintptr_t addr0 = (uintptr_t)a.logits + (base + v0) * sizeof(T);
    const int head = min((int)(((16 - (addr0 & 15)) & 15) / sizeof(T)), v1 - v0);
    if ((int)threadIdx.x < head) count += score<T>(a.logits, base + v0 + threadIdx.x) > mine;
    const int body0 = v0 + head, n_vec = (v1 - body0) / kPer;
    const u32x4* vec = reinterpret_cast<const u32x4*>(reinterpret_cast<const T*>(a.logits) + base + body0);
    for (int k = threadIdx.x; k < n_vec; k += kThreads) {
        const u32x4 w = __builtin_nontemporal_load(vec + k);  // a row is streamed once
        // elements go to scalars first: __builtin_bit_cast applied to a vector-element expression was
        // seen to read element 0 for every index
        const uint32_t w0 = w[0], w1 = w[1], w2 = w[2], w3 = w[3];
        if constexpr (sizeof(T) == 4) {
            count += (__builtin_bit_cast(float, w0) > mine) + (__builtin_bit_cast(float, w1) > mine) +
                     (__builtin_bit_cast(float, w2) > mine) + (__builtin_bit_cast(float, w3) > mine);
        } else {
            count += above_pair(w0, mine) + above_pair(w1, mine) + above_pair(w2, mine) + above_pair(w3, mine);
        }
    }
    const int tail0 = body0 + n_vec * kPer;
    if (tail0 + (int)threadIdx.x < v1) count += score<T>(a.logits, base + tail0 + threadIdx.x) > mine;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) count += __shfl_xor(count, o, kWave);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = count;
    __syncthreads();
    if (threadIdx.x == 0) {
        int total = 0;
#pragma unroll
        for (int w = 0; w < kThreads / 64; ++w) total += part[w];
        if (total) atomicAdd(a.rank + d, total);
    }
}

__global__ __launch_bounds__(kThreads) void rank_mask_kernel(RankArgs a) {
    const int row = blockIdx.x * kThreads + threadIdx.x;
    if (row >= a.N_cap || row >= a.cu_q[a.B]) return;
    const int i = owner(a.cu_q, a.B, row);
    const int j = row - a.cu_q[i];  // the row's input is draft j - 1 of the request
    uint8_t keep = 1;
    if (j >= 1 && j - 1 < a.cu_d[i + 1] - a.cu_d[i]) keep = a.rank[a.cu_d[i] + j - 1] < a.K ? 1 : 0;
    a.keep[row] = keep;
}

}  // namespace
}  // namespace fsr

using namespace fsr;

extern "C" int fsr_topk_rank_check(const void* logits, const int32_t* draft_tokens, const int32_t* cu_q,
                                   const int32_t* cu_d, int32_t* rank, uint8_t* keep_mask,
                                   const fsr_rank_params* p, void* stream) {
    if (!p) return fail(FSR_EINVAL, "fsr_topk_rank_check: params is null");
    if (p->B < 0 || p->N_cap < 0 || p->D_cap < 0 || p->V <= 0 || p->K < 0 || p->reserved != 0)
        return fail(FSR_EINVAL, "fsr_topk_rank_check: B=%d N_cap=%d D_cap=%d V=%d K=%d reserved=%d", p->B, p->N_cap, p->D_cap,
                    p->V, p->K, p->reserved);
    if (p->dtype != FSR_F32 && p->dtype != FSR_BF16) return fail(FSR_EUNSUP, "fsr_topk_rank_check: dtype=%d", p->dtype);
    if (p->B == 0 || p->N_cap == 0) return FSR_OK;
    if (!logits || !cu_q || !cu_d || !keep_mask || (p->D_cap > 0 && (!draft_tokens || !rank)))
        return fail(FSR_EINVAL, "fsr_topk_rank_check: null pointer among logits/draft_tokens/cu_q/cu_d/rank/keep_mask");
    if (p->D_cap > 65535) return fail(FSR_EUNSUP, "fsr_topk_rank_check: D_cap=%d exceeds 65535 drafts per call", p->D_cap);
    if ((uintptr_t)logits & (p->dtype == FSR_F32 ? 3 : 1)) return fail(FSR_EINVAL, "fsr_topk_rank_check: logits misaligned");
    hipStream_t s = (hipStream_t)stream;
    RankArgs a;
    a.logits = logits; a.draft_tokens = draft_tokens; a.cu_q = cu_q; a.cu_d = cu_d; a.rank = rank; a.keep = keep_mask;
    a.B = p->B; a.V = p->V; a.K = p->K; a.N_cap = p->N_cap; a.D_cap = p->D_cap;
    if (p->D_cap > 0) {
        hipLaunchKernelGGL(rank_init_kernel, dim3((p->D_cap + kThreads - 1) / kThreads), dim3(kThreads), 0, s, a);
        const dim3 grid((p->V + kChunk - 1) / kChunk, p->D_cap);
        if (p->dtype == FSR_F32) hipLaunchKernelGGL(rank_count_kernel<float>, grid, dim3(kThreads), 0, s, a);
        else hipLaunchKernelGGL(rank_count_kernel<uint16_t>, grid, dim3(kThreads), 0, s, a);
    }
    hipLaunchKernelGGL(rank_mask_kernel, dim3((p->N_cap + kThreads - 1) / kThreads), dim3(kThreads), 0, s, a);
    return check_launch("fsr_topk_rank_check");
}
