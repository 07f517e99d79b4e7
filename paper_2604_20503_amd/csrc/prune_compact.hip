// prune_compact / prune_restore / frontier state kernels (integer work, bit-exact).
//
// The ragged metadata of a verification batch is a few KB (B <= a few thousand requests,
// N <= a few thousand rows), so the offsets and row maps are produced by ONE workgroup that
// walks the requests in tiles of 1024 with a running carry: latency-bound, no inter-block
// synchronisation.  The optional payload gather is the only part that moves real bytes and
// runs as a separate grid over rows with 16-byte accesses.
#include "common.hpp"
#include "device_utils.hpp"

namespace fsr {

namespace {

constexpr int kScanThreads = 1024;

// Exclusive scan of one value per thread over the block; returns the exclusive prefix and
// sets `total`.  smem must hold kScanThreads / 64 + 1 ints.
__device__ __forceinline__ int block_exclusive_scan(int v, int* smem, int& total) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int inc = wave_inclusive_scan(v);
    if (lane == 63) smem[w] = inc;
    __syncthreads();
    if (w == 0) {
        int s = lane < (kScanThreads / 64) ? smem[lane] : 0;
        int si = wave_inclusive_scan(s);
        if (lane < (kScanThreads / 64)) smem[lane] = si - s;
        if (lane == (kScanThreads / 64) - 1) smem[kScanThreads / 64] = si;
    }
    __syncthreads();
    const int base = smem[w];
    total = smem[kScanThreads / 64];
    __syncthreads();
    return base + inc - v;
}

// keep: the mask; or, when accepted_len is given instead, request i keeps its rows 0 .. accepted_len[i]
// (the survivors of an accept step; always suffix-closed) and keep_out, if not null, receives that mask.
__global__ __launch_bounds__(kScanThreads) void prune_scan_kernel(
    const uint8_t* __restrict__ keep, const int32_t* __restrict__ accepted_len, uint8_t* __restrict__ keep_out,
    const int32_t* __restrict__ cu_q, int32_t* __restrict__ new_cu_q,
    int32_t* __restrict__ new_q_lens, int32_t* __restrict__ src_row, int32_t* __restrict__ dst_row,
    int32_t* __restrict__ n_active, int32_t* __restrict__ active_ids, int B, int N_cap, int suffix_close) {
    __shared__ int smem[kScanThreads / 64 + 1];
    int row_carry = 0, act_carry = 0;
    const int N = B > 0 ? min(max(cu_q[B], 0), N_cap) : 0;
    for (int base = 0; base < B; base += kScanThreads) {
        const int i = base + threadIdx.x;
        int kept = 0, r0 = 0, r1 = 0;
        if (i < B) {
            r0 = min(max(cu_q[i], 0), N_cap);  // offsets beyond the allocated rows are cut off
            r1 = min(max(cu_q[i + 1], r0), N_cap);
            if (accepted_len) {
                kept = min(max(accepted_len[i] + 1, 0), r1 - r0);
            } else if (suffix_close) {
                int r = r0;
                while (r < r1 && keep[r] != 0) ++r;
                kept = r - r0;
            } else {
                for (int r = r0; r < r1; ++r) kept += keep[r] != 0;
            }
        }
        int tile_rows, tile_act;
        const int off = row_carry + block_exclusive_scan(kept, smem, tile_rows);
        const int aoff = act_carry + block_exclusive_scan(kept > 0 ? 1 : 0, smem, tile_act);
        if (i < B) {
            new_cu_q[i] = off;
            new_q_lens[i] = kept;
            if (kept > 0) active_ids[aoff] = i;
            int o = off;
            for (int r = r0; r < r1; ++r) {
                const bool k = suffix_close ? (r - r0 < kept) : (keep[r] != 0);
                if (keep_out) keep_out[r] = k ? 1 : 0;
                if (k) {
                    src_row[o] = r;
                    dst_row[r] = o;
                    ++o;
                } else {
                    dst_row[r] = -1;
                }
            }
        }
        row_carry += tile_rows;
        act_carry += tile_act;
    }
    if (threadIdx.x == 0) {
        new_cu_q[B] = row_carry;
        n_active[0] = act_carry;
    }
    for (int r = row_carry + threadIdx.x; r < N_cap; r += kScanThreads) src_row[r] = -1;
    for (int r = N + threadIdx.x; r < N_cap; r += kScanThreads) dst_row[r] = -1;
    for (int a = act_carry + threadIdx.x; a < B; a += kScanThreads) active_ids[a] = -1;
}

// payload_out[r'] = payload_in[src_row[r']] for r' < n_new[0]; one block per output row slice.
template <typename VecT>
__global__ __launch_bounds__(256) void gather_rows_kernel(const VecT* __restrict__ in, VecT* __restrict__ out,
                                                          const int32_t* __restrict__ src_row,
                                                          const int32_t* __restrict__ n_new, size_t row_vecs,
                                                          int N_cap) {
    const int n = min(n_new[0], N_cap);
    for (int r = blockIdx.x; r < n; r += gridDim.x) {
        const int s = src_row[r];
        if (s < 0 || s >= N_cap) continue;
        const VecT* src = in + (size_t)s * row_vecs;
        VecT* dst = out + (size_t)r * row_vecs;
        for (size_t v = (size_t)blockIdx.y * blockDim.x + threadIdx.x; v < row_vecs; v += (size_t)gridDim.y * blockDim.x)
            dst[v] = src[v];
    }
}

// out[src_row[r']] = compact[r'] for r' < n_new[0]; rows of `out` that no r' maps to keep their contents.
template <typename VecT>
__global__ __launch_bounds__(256) void scatter_rows_kernel(const VecT* __restrict__ compact, VecT* __restrict__ out,
                                                           const int32_t* __restrict__ src_row,
                                                           const int32_t* __restrict__ n_new, size_t row_vecs,
                                                           int N_cap) {
    const int n = min(n_new[0], N_cap);
    for (int r = blockIdx.x; r < n; r += gridDim.x) {
        const int d = src_row[r];
        if (d < 0 || d >= N_cap) continue;
        const VecT* src = compact + (size_t)r * row_vecs;
        VecT* dst = out + (size_t)d * row_vecs;
        for (size_t v = (size_t)blockIdx.y * blockDim.x + threadIdx.x; v < row_vecs; v += (size_t)gridDim.y * blockDim.x)
            dst[v] = src[v];
    }
}

template <typename VecT>
__global__ __launch_bounds__(256) void restore_rows_kernel(const VecT* __restrict__ compact,
                                                           const int32_t* __restrict__ dst_row,
                                                           VecT* __restrict__ restored, uint8_t* __restrict__ has_value,
                                                           size_t row_vecs, int N, VecT pad) {
    for (int r = blockIdx.x; r < N; r += gridDim.x) {
        const int s = dst_row[r];
        VecT* dst = restored + (size_t)r * row_vecs;
        if (s >= 0) {
            const VecT* src = compact + (size_t)s * row_vecs;
            for (size_t v = (size_t)blockIdx.y * blockDim.x + threadIdx.x; v < row_vecs; v += (size_t)gridDim.y * blockDim.x)
                dst[v] = src[v];
        } else {
            for (size_t v = (size_t)blockIdx.y * blockDim.x + threadIdx.x; v < row_vecs; v += (size_t)gridDim.y * blockDim.x)
                dst[v] = pad;
        }
        if (has_value && blockIdx.y == 0 && threadIdx.x == 0) has_value[r] = s >= 0 ? 1 : 0;
    }
}

// keep[r] = 1 for rows 0 .. accepted_len[i] of request i (the rows whose tokens stay committed after
// the accept step: the last committed token and the accepted drafts), 0 for the rejected suffix.
__global__ void survivor_mask_kernel(const int32_t* __restrict__ accepted_len, const int32_t* __restrict__ cu_q,
                                     uint8_t* __restrict__ keep, int B, int N_cap) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= B) return;
    const int r0 = min(max(cu_q[i], 0), N_cap), r1 = min(max(cu_q[i + 1], r0), N_cap);
    const int n = accepted_len[i];
    for (int r = r0; r < r1; ++r) keep[r] = (r - r0 <= n) ? 1 : 0;
}

__global__ void frontier_init_kernel(const int32_t* __restrict__ spec_lens, int32_t* pos, int32_t* active,
                                     int32_t* n_out, int32_t* acc_total, int32_t* out_tokens, int B, int out_stride) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= B) return;
    pos[i] = 0;
    active[i] = 1;
    n_out[i] = 0;
    acc_total[i] = 0;
    for (int s = 0; s < out_stride; ++s) out_tokens[(size_t)i * out_stride + s] = -1;
}

__global__ void frontier_plan_kernel(const int32_t* __restrict__ ctx_lens, const int32_t* __restrict__ spec_lens,
                                     const int32_t* __restrict__ cu_q, const int32_t* __restrict__ cu_d,
                                     const int32_t* __restrict__ pos, const int32_t* __restrict__ active,
                                     const int32_t* __restrict__ chunk_len, uint8_t* __restrict__ t_mask,
                                     uint8_t* __restrict__ d_mask, int32_t* __restrict__ chunk_ctx, int B,
                                     int N_t_cap, int N_d_cap) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= B) return;
    const int t0 = cu_q[i], t1 = min(cu_q[i + 1], N_t_cap), d0 = cu_d[i], d1 = min(cu_d[i + 1], N_d_cap);
    const int s = spec_lens[i], p = pos[i];
    int nk = 0, nt = 0;
    if (active[i]) {
        nk = max(0, min(chunk_len[i], s - p));
        // the bonus row rides with the chunk that verifies the last draft (or is the only
        // row of a request without drafts)
        const bool last = (p + nk == s) && (nk > 0 || s == 0);
        nt = nk + (last ? 1 : 0);
    }
    for (int r = t0; r < t1; ++r) t_mask[r] = (r - t0 >= p && r - t0 < p + nt) ? 1 : 0;
    for (int r = d0; r < d1; ++r) d_mask[r] = (r - d0 >= p && r - d0 < p + nk) ? 1 : 0;
    chunk_ctx[i] = ctx_lens[i] + p;
}

__global__ void frontier_commit_kernel(const int32_t* __restrict__ spec_lens, const int32_t* __restrict__ chunk_len,
                                       const int32_t* __restrict__ accepted_len, const int32_t* __restrict__ n_emitted,
                                       const int32_t* __restrict__ emitted, int emitted_stride, int32_t* pos,
                                       int32_t* active, int32_t* n_out, int32_t* acc_total, int32_t* out_tokens, int B,
                                       int out_stride) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= B) return;
    if (!active[i]) return;
    const int s = spec_lens[i], p = pos[i];
    const int nk = max(0, min(chunk_len[i], s - p));
    const int ne = max(0, min(n_emitted[i], emitted_stride));
    int o = n_out[i];
    for (int e = 0; e < ne && o < out_stride; ++e, ++o) out_tokens[(size_t)i * out_stride + o] = emitted[(size_t)i * emitted_stride + e];
    n_out[i] = o;
    const int a = accepted_len[i];
    acc_total[i] += max(a, 0);
    pos[i] = p + nk;
    if (a < nk || p + nk >= s) active[i] = 0;
}

template <typename F>
int launch_by_width(size_t row_bytes, const void* a, const void* b, F&& f) {
    const uintptr_t bits = (uintptr_t)a | (uintptr_t)b | (uintptr_t)row_bytes;
    if ((bits & 15) == 0) return f(uint4{}, row_bytes / 16);
    return f(uint32_t{}, row_bytes / 4);
}

}  // namespace
}  // namespace fsr

using namespace fsr;

namespace {
// Both compaction entry points: the kept rows come from keep_mask, or from accepted_len (then keep_out, nullable,
// receives the mask and the rule is suffix-closed by construction).
int compact_call(const char* who, const uint8_t* keep_mask, const int32_t* accepted_len, uint8_t* keep_out, const int32_t* cu_q,
                 int32_t* new_cu_q, int32_t* new_q_lens, int32_t* src_row, int32_t* dst_row, int32_t* n_active,
                 int32_t* active_ids, const void* payload_in, void* payload_out, size_t row_bytes, const fsr_prune_params* p,
                 void* stream) {
    if (!p) return fail(FSR_EINVAL, "%s: params is null", who);
    if (p->B < 0 || p->N_cap < 0 || p->reserved != 0) return fail(FSR_EINVAL, "%s: B=%d N_cap=%d reserved=%d", who, p->B, p->N_cap, p->reserved);
    if (!cu_q || !new_cu_q || !n_active) return fail(FSR_EINVAL, "%s: cu_q/new_cu_q/n_active is null", who);
    if (p->B > 0 && (!new_q_lens || !active_ids)) return fail(FSR_EINVAL, "%s: new_q_lens/active_ids is null", who);
    if (p->N_cap > 0 && ((!keep_mask && !accepted_len) || !src_row || !dst_row))
        return fail(FSR_EINVAL, "%s: %s/src_row/dst_row is null", who, accepted_len || keep_out ? "accepted_len" : "keep_mask");
    if ((payload_in == nullptr) != (payload_out == nullptr)) return fail(FSR_EINVAL, "%s: payload_in and payload_out must both be given or both be null", who);
    if (payload_in && (row_bytes == 0 || row_bytes % 4 != 0)) return fail(FSR_ESHAPE, "%s: row_bytes=%zu must be a positive multiple of 4", who, row_bytes);
    if (payload_in && payload_in == payload_out) return fail(FSR_EINVAL, "%s: payload gather cannot run in place", who);
    hipStream_t s = (hipStream_t)stream;
    hipLaunchKernelGGL(prune_scan_kernel, dim3(1), dim3(kScanThreads), 0, s, keep_mask, accepted_len, keep_out, cu_q, new_cu_q,
                       new_q_lens, src_row, dst_row, n_active, active_ids, p->B, p->N_cap, accepted_len ? 1 : p->suffix_close);
    int rc = check_launch("prune_scan_kernel");
    if (rc != FSR_OK) return rc;
    if (payload_in && p->N_cap > 0) {
        const int N_cap = p->N_cap;
        rc = launch_by_width(row_bytes, payload_in, payload_out, [&](auto tag, size_t row_vecs) {
            using VecT = decltype(tag);
            const unsigned gy = (unsigned)std::min<size_t>(std::max<size_t>(1, (row_vecs + 255) / 256), 64);
            const unsigned gx = (unsigned)std::min(N_cap, 65535);
            hipLaunchKernelGGL(gather_rows_kernel<VecT>, dim3(gx, gy), dim3(256), 0, s, (const VecT*)payload_in,
                               (VecT*)payload_out, src_row, new_cu_q + p->B, row_vecs, N_cap);
            return check_launch("gather_rows_kernel");
        });
    }
    return rc;
}
}  // namespace

extern "C" int fsr_prune_compact(const uint8_t* keep_mask, const int32_t* cu_q, int32_t* new_cu_q,
                                 int32_t* new_q_lens, int32_t* src_row, int32_t* dst_row, int32_t* n_active,
                                 int32_t* active_ids, const void* payload_in, void* payload_out, size_t row_bytes,
                                 const fsr_prune_params* p, void* stream) {
    return compact_call("fsr_prune_compact", keep_mask, nullptr, nullptr, cu_q, new_cu_q, new_q_lens, src_row, dst_row, n_active,
                        active_ids, payload_in, payload_out, row_bytes, p, stream);
}

extern "C" int fsr_survivor_compact(const int32_t* accepted_len, const int32_t* cu_q, uint8_t* keep_mask, int32_t* new_cu_q,
                                    int32_t* new_q_lens, int32_t* src_row, int32_t* dst_row, int32_t* n_active,
                                    int32_t* active_ids, const void* payload_in, void* payload_out, size_t row_bytes,
                                    const fsr_prune_params* p, void* stream) {
    if (p && p->B > 0 && !accepted_len) return fail(FSR_EINVAL, "fsr_survivor_compact: accepted_len is null");
    return compact_call("fsr_survivor_compact", nullptr, accepted_len, keep_mask, cu_q, new_cu_q, new_q_lens, src_row, dst_row,
                        n_active, active_ids, payload_in, payload_out, row_bytes, p, stream);
}

extern "C" int fsr_prune_restore(const void* compact, const int32_t* dst_row, void* restored, uint8_t* has_value,
                                 size_t row_bytes, int32_t N, uint32_t pad_word, void* stream) {
    if (N < 0) return fail(FSR_EINVAL, "fsr_prune_restore: N=%d", N);
    if (N == 0) return FSR_OK;
    if (!compact || !dst_row || !restored) return fail(FSR_EINVAL, "fsr_prune_restore: null pointer");
    if (row_bytes == 0 || row_bytes % 4 != 0) return fail(FSR_ESHAPE, "fsr_prune_restore: row_bytes=%zu must be a positive multiple of 4", row_bytes);
    if (compact == restored) return fail(FSR_EINVAL, "fsr_prune_restore: cannot run in place");
    hipStream_t s = (hipStream_t)stream;
    return launch_by_width(row_bytes, compact, restored, [&](auto tag, size_t row_vecs) {
        using VecT = decltype(tag);
        VecT pad;
        if constexpr (sizeof(VecT) == 16) pad = uint4{pad_word, pad_word, pad_word, pad_word};
        else pad = pad_word;
        const unsigned gy = (unsigned)std::min<size_t>(std::max<size_t>(1, (row_vecs + 255) / 256), 64);
        const unsigned gx = (unsigned)std::min(N, 65535);
        hipLaunchKernelGGL(restore_rows_kernel<VecT>, dim3(gx, gy), dim3(256), 0, s, (const VecT*)compact, dst_row,
                           (VecT*)restored, has_value, row_vecs, N, pad);
        return check_launch("restore_rows_kernel");
    });
}

extern "C" int fsr_prune_scatter(const void* compact, const int32_t* src_row, const int32_t* n_rows, void* out,
                                 size_t row_bytes, int32_t N_cap, void* stream) {
    if (N_cap < 0) return fail(FSR_EINVAL, "fsr_prune_scatter: N_cap=%d", N_cap);
    if (N_cap == 0) return FSR_OK;
    if (!compact || !src_row || !n_rows || !out) return fail(FSR_EINVAL, "fsr_prune_scatter: null pointer");
    if (row_bytes == 0 || row_bytes % 4 != 0) return fail(FSR_ESHAPE, "fsr_prune_scatter: row_bytes=%zu must be a positive multiple of 4", row_bytes);
    if (compact == out) return fail(FSR_EINVAL, "fsr_prune_scatter: cannot run in place");
    hipStream_t s = (hipStream_t)stream;
    return launch_by_width(row_bytes, compact, out, [&](auto tag, size_t row_vecs) {
        using VecT = decltype(tag);
        const unsigned gy = (unsigned)std::min<size_t>(std::max<size_t>(1, (row_vecs + 255) / 256), 64);
        const unsigned gx = (unsigned)std::min(N_cap, 65535);
        hipLaunchKernelGGL(scatter_rows_kernel<VecT>, dim3(gx, gy), dim3(256), 0, s, (const VecT*)compact, (VecT*)out,
                           src_row, n_rows, row_vecs, N_cap);
        return check_launch("scatter_rows_kernel");
    });
}

extern "C" int fsr_survivor_mask(const int32_t* accepted_len, const int32_t* cu_q, uint8_t* keep_mask, int32_t B,
                                 int32_t N_cap, void* stream) {
    if (B < 0 || N_cap < 0) return fail(FSR_EINVAL, "fsr_survivor_mask: B=%d N_cap=%d", B, N_cap);
    if (B == 0 || N_cap == 0) return FSR_OK;
    if (!accepted_len || !cu_q || !keep_mask) return fail(FSR_EINVAL, "fsr_survivor_mask: null pointer");
    hipLaunchKernelGGL(survivor_mask_kernel, dim3((B + 255) / 256), dim3(256), 0, (hipStream_t)stream, accepted_len, cu_q,
                       keep_mask, B, N_cap);
    return check_launch("survivor_mask_kernel");
}

extern "C" int fsr_frontier_init(const int32_t* spec_lens, int32_t* pos, int32_t* active, int32_t* n_out,
                                 int32_t* acc_total, int32_t* out_tokens, int32_t B, int32_t out_stride, void* stream) {
    if (B < 0 || out_stride < 0) return fail(FSR_EINVAL, "fsr_frontier_init: B=%d out_stride=%d", B, out_stride);
    if (B == 0) return FSR_OK;
    if (!spec_lens || !pos || !active || !n_out || !acc_total || !out_tokens) return fail(FSR_EINVAL, "fsr_frontier_init: null pointer");
    hipLaunchKernelGGL(frontier_init_kernel, dim3((B + 255) / 256), dim3(256), 0, (hipStream_t)stream, spec_lens, pos, active,
                       n_out, acc_total, out_tokens, B, out_stride);
    return check_launch("frontier_init_kernel");
}

extern "C" int fsr_frontier_plan(const int32_t* ctx_lens, const int32_t* spec_lens, const int32_t* cu_q,
                                 const int32_t* cu_d, const int32_t* pos, const int32_t* active,
                                 const int32_t* chunk_len, uint8_t* t_mask, uint8_t* d_mask, int32_t* chunk_ctx,
                                 int32_t B, int32_t N_t_cap, int32_t N_d_cap, void* stream) {
    if (B < 0 || N_t_cap < 0 || N_d_cap < 0) return fail(FSR_EINVAL, "fsr_frontier_plan: B=%d N_t_cap=%d N_d_cap=%d", B, N_t_cap, N_d_cap);
    if (B == 0) return FSR_OK;
    if (!ctx_lens || !spec_lens || !cu_q || !cu_d || !pos || !active || !chunk_len || !chunk_ctx) return fail(FSR_EINVAL, "fsr_frontier_plan: null pointer");
    if ((N_t_cap > 0 && !t_mask) || (N_d_cap > 0 && !d_mask)) return fail(FSR_EINVAL, "fsr_frontier_plan: mask is null");
    hipLaunchKernelGGL(frontier_plan_kernel, dim3((B + 255) / 256), dim3(256), 0, (hipStream_t)stream, ctx_lens, spec_lens, cu_q,
                       cu_d, pos, active, chunk_len, t_mask, d_mask, chunk_ctx, B, N_t_cap, N_d_cap);
    return check_launch("frontier_plan_kernel");
}

extern "C" int fsr_frontier_commit(const int32_t* spec_lens, const int32_t* chunk_len, const int32_t* accepted_len,
                                   const int32_t* n_emitted, const int32_t* emitted, int32_t emitted_stride,
                                   int32_t* pos, int32_t* active, int32_t* n_out, int32_t* acc_total,
                                   int32_t* out_tokens, int32_t B, int32_t out_stride, void* stream) {
    if (B < 0 || emitted_stride < 1 || out_stride < 1) return fail(FSR_EINVAL, "fsr_frontier_commit: B=%d emitted_stride=%d out_stride=%d", B, emitted_stride, out_stride);
    if (B == 0) return FSR_OK;
    if (!spec_lens || !chunk_len || !accepted_len || !n_emitted || !emitted || !pos || !active || !n_out || !acc_total || !out_tokens)
        return fail(FSR_EINVAL, "fsr_frontier_commit: null pointer");
    hipLaunchKernelGGL(frontier_commit_kernel, dim3((B + 255) / 256), dim3(256), 0, (hipStream_t)stream, spec_lens, chunk_len,
                       accepted_len, n_emitted, emitted, emitted_stride, pos, active, n_out, acc_total, out_tokens, B, out_stride);
    return check_launch("frontier_commit_kernel");
}
