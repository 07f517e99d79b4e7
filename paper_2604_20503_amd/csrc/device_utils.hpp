// Wavefront-level (64 lanes) reductions and scans, and the arrival counter several kernels use to
// find out which workgroup is the last of a group to finish.
#pragma once
#include <hip/hip_runtime.h>

namespace fsr {

constexpr int kWave = 64;

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
    return v;
}

__device__ __forceinline__ int wave_min_i(int v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = min(v, __shfl_xor(v, o, kWave));
    return v;
}

__device__ __forceinline__ int wave_max_i(int v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = max(v, __shfl_xor(v, o, kWave));
    return v;
}

// Inclusive scan across the 64 lanes of a wave.
template <typename T>
__device__ __forceinline__ T wave_inclusive_scan(T v) {
    const int lane = threadIdx.x & (kWave - 1);
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
        T up = __shfl_up(v, o, kWave);
        if (lane >= o) v += up;
    }
    return v;
}

// Count one more arrival on a 64-bit word that holds (call id << 16 | count).  A word left by another
// call (or never written) counts as zero, so the memory it lives in needs no clearing between calls
// and HIP-graph replays work.  Returns the count including this arrival.  Device scope.
__device__ __forceinline__ int count_arrival(unsigned long long* word, unsigned long long call_id) {
    unsigned long long seen = __atomic_load_n(word, __ATOMIC_RELAXED);
    for (;;) {
        const unsigned long long have = (seen >> 16) == call_id ? (seen & 0xffffu) : 0u;
        const unsigned long long want = (call_id << 16) | (have + 1);
        const unsigned long long prev = atomicCAS(word, seen, want);
        if (prev == seen) return (int)(have + 1);
        seen = prev;
    }
}

}  // namespace fsr
