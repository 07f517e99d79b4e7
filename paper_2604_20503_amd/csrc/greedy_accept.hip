// Greedy (temperature 0) mode of fsr_spec_accept: Sec. 2.1's accept-until-first-mismatch rule with
// an arg-max target.  A draft is accepted iff it is the arg-max token of its target row (lowest id
// among equal maxima); the token after the accepted run is the arg-max of the next target row.
//
// The cost is one streaming pass over the target rows (4 V bytes each).  All rows are reduced in
// parallel (a request's rows behind its first mismatch are read although not needed: the
// alternative, row after row, would put one memory round trip per accepted draft on the critical
// path).  greedy_argmax_kernel: grid (16 KB chunks, rows); every workgroup folds its chunk into a
// 64-bit key (value made order-preserving << 32 | ~index) and merges it into the row's key with one
// atomic max, which yields the largest value and, among equals, the lowest index.
#include <cstdint>

#include "common.hpp"
#include "device_utils.hpp"
#include "greedy_accept.hpp"

namespace fsr {
namespace {

constexpr int kThreads = 256;
constexpr int kChunk = 4096;  // scores per workgroup

typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;

// fp32 bits -> unsigned integer with the same order (-0 and +0 map to the same key; a NaN never wins
// against a number: it takes the key of minus infinity).
__device__ __forceinline__ uint32_t ordered_bits(uint32_t b) {
    if ((b << 1) == 0) b = 0;  // -0 -> +0
    if ((b & 0x7fffffffu) > 0x7f800000u) b = 0xff800000u;  // NaN -> -inf
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
__device__ __forceinline__ unsigned long long make_key(uint32_t bits, int idx) {
    return ((unsigned long long)ordered_bits(bits) << 32) | (uint32_t)(0xffffffffu - (uint32_t)idx);
}
__device__ __forceinline__ unsigned long long wave_max_u64(unsigned long long k) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const uint32_t lo = __shfl_xor((uint32_t)k, o, kWave), hi = __shfl_xor((uint32_t)(k >> 32), o, kWave);
        const unsigned long long other = ((unsigned long long)hi << 32) | lo;
        k = other > k ? other : k;
    }
    return k;
}

__global__ __launch_bounds__(kThreads) void greedy_init_kernel(unsigned long long* keys, int n) {
    const int r = blockIdx.x * kThreads + threadIdx.x;
    if (r < n) keys[r] = 0ull;
}

__global__ __launch_bounds__(kThreads) void greedy_argmax_kernel(const float* __restrict__ target,
                                                                 const int32_t* __restrict__ cu_t,
                                                                 const int32_t* __restrict__ t_rows,
                                                                 unsigned long long* keys, int B, int V, int R_cap) {
    __shared__ unsigned long long part[kThreads / 64];
    const int r = blockIdx.y;  // call-row on the target side
    if (r >= R_cap || r >= cu_t[B]) return;
    const long long row = t_rows ? t_rows[r] : r;
    const float* z = target + (size_t)row * V;
    const int v0 = blockIdx.x * kChunk, v1 = min(v0 + kChunk, V);
    unsigned long long best = 0ull;
    // peel up to the first 16-byte boundary, then 16-byte loads, then the tail
    const uintptr_t addr0 = (uintptr_t)(z + v0);
    const int head = min((int)(((16 - (addr0 & 15)) & 15) / 4), v1 - v0);
    if ((int)threadIdx.x < head) {
        const int v = v0 + threadIdx.x;
        best = make_key(__builtin_bit_cast(uint32_t, z[v]), v);
    }
    const int body0 = v0 + head, n_vec = (v1 - body0) / 4;
    const u32x4* vec = reinterpret_cast<const u32x4*>(z + body0);
    for (int k = threadIdx.x; k < n_vec; k += kThreads) {
        const u32x4 w = __builtin_nontemporal_load(vec + k);  // a row is streamed once
        const uint32_t w0 = w[0], w1 = w[1], w2 = w[2], w3 = w[3];
        const int v = body0 + 4 * k;
        unsigned long long c = make_key(w0, v);
        const unsigned long long c1 = make_key(w1, v + 1), c2 = make_key(w2, v + 2), c3 = make_key(w3, v + 3);
        c = c1 > c ? c1 : c;
        c = c2 > c ? c2 : c;
        c = c3 > c ? c3 : c;
        best = c > best ? c : best;
    }
    const int tail0 = body0 + n_vec * 4;
    if (tail0 + (int)threadIdx.x < v1) {
        const int v = tail0 + threadIdx.x;
        const unsigned long long c = make_key(__builtin_bit_cast(uint32_t, z[v]), v);
        best = c > best ? c : best;
    }
    best = wave_max_u64(best);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = best;
    __syncthreads();
    if (threadIdx.x == 0) {
#pragma unroll
        for (int w = 1; w < kThreads / 64; ++w) best = part[w] > best ? part[w] : best;
        atomicMax(keys + r, best);
    }
}

__global__ __launch_bounds__(kThreads) void greedy_decide_kernel(const int32_t* __restrict__ draft_tokens,
                                                                 const int32_t* __restrict__ cu_t,
                                                                 const int32_t* __restrict__ cu_d,
                                                                 const int32_t* __restrict__ d_rows,
                                                                 const unsigned long long* __restrict__ keys,
                                                                 int32_t* accepted_len, int32_t* n_emitted,
                                                                 int32_t* emitted, int B, int S_max, int R_cap) {
    const int i = blockIdx.x * kThreads + threadIdx.x;
    if (i >= B) return;
    const int d_i = cu_d[i + 1] - cu_d[i], t_i = cu_t[i + 1] - cu_t[i];
    int32_t* em = emitted + (size_t)i * (S_max + 1);
    for (int s = 0; s <= S_max; ++s) em[s] = -1;
    // a request whose row counts do not fit the call is flagged, not processed
    if (d_i < 0 || d_i > S_max || t_i < d_i || t_i > d_i + 1 || cu_t[i] < 0 || cu_t[i] + t_i > R_cap) {
        accepted_len[i] = -1;
        n_emitted[i] = -1;
        return;
    }
    auto choice = [&](int n) { return (int)(0xffffffffu - (uint32_t)keys[cu_t[i] + n]); };
    int n = 0, tok = -1;
    while (n < d_i) {
        const long long dr = d_rows ? d_rows[cu_d[i] + n] : cu_d[i] + n;
        const int c = choice(n);
        if (draft_tokens[dr] != c) {
            tok = c;
            break;
        }
        em[n] = c;
        ++n;
    }
    if (n == d_i && t_i == d_i + 1) tok = choice(d_i);
    if (tok >= 0) em[n] = tok;
    accepted_len[i] = n;
    n_emitted[i] = n + (tok >= 0 ? 1 : 0);
}

}  // namespace

size_t greedy_workspace_bytes(const fsr_accept_params& p) {
    return align_up((size_t)p.B * (size_t)(p.S_max + 1) * sizeof(unsigned long long), 256);
}

int greedy_accept_launch(const float* target, const int32_t* draft_tokens, const int32_t* cu_t, const int32_t* cu_d,
                         const int32_t* t_rows, const int32_t* d_rows, int32_t* accepted_len, int32_t* n_emitted,
                         int32_t* emitted, const fsr_accept_params& p, void* workspace, hipStream_t s) {
    unsigned long long* keys = (unsigned long long*)workspace;
    const int R_cap = p.B * (p.S_max + 1);
    int rc;
    hipLaunchKernelGGL(greedy_init_kernel, dim3((R_cap + kThreads - 1) / kThreads), dim3(kThreads), 0, s, keys, R_cap);
    if ((rc = check_launch("greedy_init_kernel")) != FSR_OK) return rc;
    hipLaunchKernelGGL(greedy_argmax_kernel, dim3((p.V + kChunk - 1) / kChunk, R_cap), dim3(kThreads), 0, s, target, cu_t,
                       t_rows, keys, p.B, p.V, R_cap);
    if ((rc = check_launch("greedy_argmax_kernel")) != FSR_OK) return rc;
    hipLaunchKernelGGL(greedy_decide_kernel, dim3((p.B + kThreads - 1) / kThreads), dim3(kThreads), 0, s, draft_tokens, cu_t,
                       cu_d, d_rows, keys, accepted_len, n_emitted, emitted, p.B, p.S_max, R_cap);
    return check_launch("greedy_decide_kernel");
}

}  // namespace fsr
