// Measurement aid: a plain streaming read of a device buffer, the yardstick next to which the
// attention kernel's achieved HBM rate is reported (what one launch of trivially parallel 16-byte
// loads draws from memory on this device).  Not part of the verification path.
#include "common.hpp"

namespace fsr {
namespace {

typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;
constexpr int kProbeThreads = 256;
constexpr int kProbeInFlight = 8;  // 16-byte loads a thread keeps in flight

// Workgroup g reads the chunks g, g + grid, ...; a chunk is kProbeInFlight blocks of 4 KB, thread t taking
// 16 bytes out of each block.  SCATTER: block b of the sequence is block (b * odd constant) mod n_blocks of
// the buffer (n_blocks a power of two: a permutation), i.e. 4 KB pieces in scattered order -- the granularity
// at which a paged KV cache with 16-token pages hands out the K or V bytes of one head.  The XOR of everything
// read goes to sink[workgroup], so that no load can be dropped.
// ROWS (with SCATTER): a wave reads "its" 4 KB blocks the way the attention kernel reads a page of K -- 16
// rows of 256 bytes, one load taking 64 bytes of every row (lane -> row lane % 16, 16 bytes at 16 * (lane /
// 16) + 64 * load) -- instead of 1 KB of consecutive bytes per load.
template <bool SCATTER, bool ROWS>
__global__ __launch_bounds__(kProbeThreads) void hbm_read_probe_kernel(const u32x4* __restrict__ src, size_t n_chunks,
                                                                      unsigned long long* __restrict__ sink) {
    u32x4 acc = u32x4{0u, 0u, 0u, 0u};
    const size_t mask = n_chunks * kProbeInFlight - 1;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    for (size_t c = blockIdx.x; c < n_chunks; c += gridDim.x) {
        u32x4 v[kProbeInFlight];
#pragma unroll
        for (int k = 0; k < kProbeInFlight; ++k) {
            if (ROWS) {
                // the chunk's 8 blocks: wave w takes blocks 2 w and 2 w + 1, four loads each
                size_t blk = ((c * kProbeInFlight + 2 * w + (k >> 2)) * 0x9E3779B97F4A7C15ull) & mask;
                v[k] = __builtin_nontemporal_load(src + blk * kProbeThreads + (lane & 15) * 16 + (lane >> 4) + 4 * (k & 3));
            } else {
                size_t blk = c * kProbeInFlight + k;
                if (SCATTER) blk = (blk * 0x9E3779B97F4A7C15ull) & mask;
                v[k] = __builtin_nontemporal_load(src + blk * kProbeThreads + threadIdx.x);
            }
        }
#pragma unroll
        for (int k = 0; k < kProbeInFlight; ++k) acc ^= v[k];
    }
    unsigned long long x = ((unsigned long long)(acc[0] ^ acc[2]) << 32) | (acc[1] ^ acc[3]);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x ^= __shfl_xor(x, off, 64);
    __shared__ unsigned long long part[kProbeThreads / 64];
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = x;
    __syncthreads();
    if (threadIdx.x == 0) sink[blockIdx.x] = part[0] ^ part[1] ^ part[2] ^ part[3];
}

}  // namespace
}  // namespace fsr

extern "C" int fsr_hbm_read_probe(const void* src, size_t bytes, unsigned long long* sink, int workgroups, int scatter_4k, void* stream) {
    using namespace fsr;
    constexpr size_t kChunk = (size_t)kProbeInFlight * kProbeThreads * 16;
    if (!src || !sink) return fail(FSR_EINVAL, "fsr_hbm_read_probe: null pointer");
    if (((uintptr_t)src & 15) != 0) return fail(FSR_EINVAL, "fsr_hbm_read_probe: src must be 16-byte aligned");
    if (bytes < kChunk || bytes % kChunk != 0)
        return fail(FSR_EINVAL, "fsr_hbm_read_probe: bytes=%zu must be a positive multiple of %zu", bytes, kChunk);
    if (workgroups <= 0 || workgroups > 65535) return fail(FSR_EINVAL, "fsr_hbm_read_probe: workgroups=%d", workgroups);
    if (scatter_4k && (bytes & (bytes - 1)) != 0) return fail(FSR_EINVAL, "fsr_hbm_read_probe: scattered order needs a power-of-two size, got %zu", bytes);
    if (scatter_4k == 2)
        hipLaunchKernelGGL((hbm_read_probe_kernel<true, true>), dim3(workgroups), dim3(kProbeThreads), 0, (hipStream_t)stream,
                           (const u32x4*)src, bytes / kChunk, sink);
    else if (scatter_4k)
        hipLaunchKernelGGL((hbm_read_probe_kernel<true, false>), dim3(workgroups), dim3(kProbeThreads), 0, (hipStream_t)stream,
                           (const u32x4*)src, bytes / kChunk, sink);
    else
        hipLaunchKernelGGL((hbm_read_probe_kernel<false, false>), dim3(workgroups), dim3(kProbeThreads), 0, (hipStream_t)stream,
                           (const u32x4*)src, bytes / kChunk, sink);
    return check_launch("hbm_read_probe_kernel");
}
