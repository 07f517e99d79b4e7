// verify_attention: ragged multi-query attention of every request's draft suffix over its
// paged KV cache, causal inside the suffix (Sec. 2.1 / 3.1 of the paper: the target model
// verifies all drafted tokens of a request in one pass; every request has its own
// speculative length).
//
// Fast path (bf16, D = 128, P = 16).  The op streams the KV cache once and is bound by HBM
// bandwidth, so everything is organised around reading K and V exactly once per KV head and
// keeping many bytes in flight per compute unit:
//   * work = 32-key tiles of every (request, KV head) item, laid end to end; a persistent
//     grid of one workgroup per compute unit cuts that line into equal contiguous shares
//     (stream-K), so a ragged batch loads every compute unit alike whatever the lengths are
//     and the lengths never leave the device;
//   * all G * q_len query rows that share a KV head form the N dimension of the matrix-core
//     tiles, so K/V bytes are reused across the GQA group and the suffix rows from registers;
//   * each of the 4 waves streams its own tiles with a two-tile register prefetch: K goes
//     straight from global memory into the A-operand layout of v_mfma_f32_16x16x32_bf16
//     (S^T = K Q^T, a lane reads 64 contiguous bytes of one key row), V is staged through a
//     wave-private, XOR-swizzled LDS tile and read back transposed with ds_read_b64_tr_b16
//     (O^T = V^T P^T);
//   * S^T's accumulator layout is exactly the B-operand layout P^T needs, so the softmax
//     runs in registers with two cross-lane steps per row;
//   * P is fed to the matrix cores as a bf16 hi + lo pair: the result is accurate to fp32
//     rounding instead of bf16 rounding of the probabilities;
//   * an item that lies inside one share is normalised and written directly; an item cut by
//     a share boundary leaves (max, sum, accumulator) partials -- at most two per workgroup --
//     that a small fix-up kernel combines.
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
typedef __attribute__((address_space(4))) int32_t const_i32;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;

constexpr int kD = 128;           // head dim of the fast path
constexpr int kP = 16;            // page size of the fast path
constexpr int kTile = 32;         // keys per wave tile
constexpr int kWaves = 4;
constexpr int kThreads = kWaves * 64;
constexpr int kMaxMT = 6;         // up to 96 query rows (G * rows) per pass
constexpr int kMaxB = 4096;       // requests whose tile prefix fits the LDS table
constexpr int kRedStride = kD + 4;  // padded row of the wave-merge buffer (floats)
// LDS map: [V tiles of the 4 waves | wave-merge buffer] (shared region), wave maxima and sums,
// Q^T operands, tile prefix of the requests, scan scratch
constexpr int kVTileBytes = kTile * kD * 2;
constexpr int kRedBytes = kWaves * 16 * kRedStride * 4;
constexpr int kStageBytes = kWaves * kVTileBytes > kRedBytes ? kWaves * kVTileBytes : kRedBytes;
constexpr int kMlOff = kStageBytes;
constexpr int kMlBytes = 2 * kWaves * 16 * kMaxMT * 4;
constexpr int kQOff = kMlOff + kMlBytes;          // Q^T operands of the current item: [kMaxMT * 4][64 lanes][16 B]
constexpr int kQBytes = kMaxMT * 4 * 64 * 16;
constexpr int kPrefOff = kQOff + kQBytes;
constexpr int kPrefBytes = (kMaxB + 1) * 4;
constexpr int kScanOff = kPrefOff + ((kPrefBytes + 15) / 16) * 16;
constexpr int kFastSmem = kScanOff + 64;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

struct FastArgs {
    const uint16_t* q;
    const uint16_t* k;
    const uint16_t* v;
    const int32_t* bt;
    const int32_t* ctx;
    const int32_t* cu_q;
    void* out;       // [N_cap, H_q, D] bf16 or fp32
    float* lse;      // nullable
    float* part_o;   // [nb * 2, m_cap, D]   unnormalised accumulators of cut items
    float* part_ml;  // [nb * 2, m_cap, 2]   (max in log2 units, sum)
    int B, H_q, H_kv, G, max_pages, n_pages;
    int nb;          // workgroups of the persistent grid
    int m_cap;       // rows (G * q_len) a partial slot holds = 16 * MTMAX
    int out_bf16;
    float scale_log2;
#ifdef FSR_TIMING
    long long* dbg;  // [nb][128 slots][4 waves] timestamps (100 MHz)
#endif
};

#ifdef FSR_TIMING
#define FSR_STAMP(slot) do { if ((threadIdx.x & 63) == 0) { const int w_ = threadIdx.x >> 6; a.dbg[(size_t)blockIdx.x * 512 + (slot) * 4 + w_] = wall_clock64(); } } while (0)
#else
#define FSR_STAMP(slot) do { } while (0)
#endif

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ uint16_t f32_to_bf16_rne(float x) { return __builtin_bit_cast(uint16_t, (__bf16)x); }

// Swizzled byte offset of 16-byte chunk `ch` (0..15) of key row `key` in a [32][128] bf16 tile.
__device__ __forceinline__ int vtile_off(int key, int ch) { return key * 256 + ((ch ^ ((key & 7) << 1)) << 4); }

// ---------------------------------------------------------------------------------------
// Schedule shared by the main and the fix-up kernel.
// pref[i] = number of 32-key tiles of requests 0..i-1 (per KV head); item (i, g) owns the
// flattened tiles [pref[i] * H_kv + g * nt_i, ... + nt_i).
// ---------------------------------------------------------------------------------------
__device__ void build_tile_prefix(const FastArgs& a, int* pref, int* scratch) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    int carry = 0;
    for (int base = 0; base < a.B; base += kThreads) {
        const int i = base + threadIdx.x;
        int nt = 0;
        if (i < a.B) {
            const int ql = a.cu_q[i + 1] - a.cu_q[i];
            if (ql > 0) {
                const int L = min(max(a.ctx[i], 0) + ql, a.max_pages * kP);
                nt = (L + kTile - 1) / kTile;
            }
        }
        const int inc = wave_inclusive_scan(nt);
        if (lane == 63) scratch[w] = inc;
        __syncthreads();
        int before = 0, total = 0;
#pragma unroll
        for (int k = 0; k < kWaves; ++k) {
            if (k < w) before += scratch[k];
            total += scratch[k];
        }
        if (i < a.B) pref[i] = carry + before + inc - nt;
        carry += total;
        __syncthreads();
    }
    if (threadIdx.x == 0) pref[a.B] = carry;
    __syncthreads();
}

struct Item {
    int i, g, nt, tile;  // request, KV head, tiles of the item, tile inside the item
};

__device__ __forceinline__ Item locate(const int* pref, int B, int H_kv, long long t) {
    int lo = 0, hi = B;  // largest i with pref[i] * H_kv <= t
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if ((long long)pref[mid] * H_kv <= t) lo = mid; else hi = mid;
    }
    Item it;
    it.i = lo;
    it.nt = pref[lo + 1] - pref[lo];
    const int local = (int)(t - (long long)pref[lo] * H_kv);
    it.g = local / it.nt;
    it.tile = local - it.g * it.nt;
    return it;
}

struct KVTile {
    bf16x8 k[2][4];
    s16x8 v[8];
};

// One (request, KV head) item, tiles [tile_a, tile_e), query rows j0 .. j0 + rows_g - 1.
// final_out: the tiles are the whole item -> normalise and write `out`; otherwise write a
// partial into slot `slot`.
template <int MT>
__device__ void attend_segment(const FastArgs& a, int i, int kvh, int c, int q0, int q_len, int j0, int rows_g,
                               int tile_a, int tile_e, bool final_out, int slot, char* smem, int seg_no = 0) {
    FSR_STAMP(seg_no * 5 + 2);
    // everything that is the same for the whole wave goes to scalar registers, so that the key
    // loop's page look-ups are scalar loads and never wait on the vector-memory queue
    i = __builtin_amdgcn_readfirstlane(i);
    kvh = __builtin_amdgcn_readfirstlane(kvh);
    c = __builtin_amdgcn_readfirstlane(c);
    q0 = __builtin_amdgcn_readfirstlane(q0);
    q_len = __builtin_amdgcn_readfirstlane(q_len);
    j0 = __builtin_amdgcn_readfirstlane(j0);
    rows_g = __builtin_amdgcn_readfirstlane(rows_g);
    tile_a = __builtin_amdgcn_readfirstlane(tile_a);
    tile_e = __builtin_amdgcn_readfirstlane(tile_e);
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lg = lane >> 4, li = lane & 15;
    const int G = a.G;
    const int M_g = G * rows_g;
    const int kv_total = min(c + q_len, a.max_pages * kP);  // tokens of this request in the cache
    const int kbeg = tile_a * kTile;
    const int kend = min(min(tile_e * kTile, c + j0 + rows_g), kv_total);  // keys any row of this pass may see
    char* vbuf = smem + w * kVTileBytes;

    // the block table is read-only input: reading it through the constant address space lets the
    // compiler use scalar loads for the (wave-uniform) page look-ups
    const const_i32* bt = (const const_i32*)(a.bt + (size_t)i * a.max_pages);
    // per-lane byte offsets inside a 4 KB (page, head) block: every load below is then
    // "uniform base + this offset + immediate", with no per-load address arithmetic
    const int k_lane = li * 256 + lg * 16;          // K: key li, 16 bytes at d = 8 lg (+ 32 kk)
    const int v_lane = lg * 256 + li * 16;          // V: key lg (+ 4 r), 16-byte chunk li
    const int vw_even = vtile_off(lg, li), vw_odd = vtile_off(4 + lg, li) - 4 * 256;  // LDS store offsets (+ 1024 r)
    // LDS transposed-read offsets: lane (lg, li) reads 8 bytes of key row 16 h + 4 lg + li/4 at
    // d = 16 db + 4 (li%4); after the transpose it holds keys 16 h + 4 lg + 0..3 at d = 16 db + li
    int vr_off[8];
    {
        const int r0 = 4 * lg + (li >> 2);
#pragma unroll
        for (int db = 0; db < 8; ++db) vr_off[db] = vtile_off(r0, 2 * db + ((li & 3) >> 1)) + (li & 1) * 8;
    }
    const size_t page_bytes = (size_t)a.H_kv * kP * kD * 2;
    const char* k_head = reinterpret_cast<const char*>(a.k) + (size_t)kvh * kP * kD * 2;
    const char* v_head = reinterpret_cast<const char*>(a.v) + (size_t)kvh * kP * kD * 2;

    // this wave's tiles: keys kb0 + t * kStep, t = 0 .. nw-1
    constexpr int kStep = kWaves * kTile;
    const int kb0 = kbeg + w * kTile;
    const int nw = kb0 < kend ? (kend - kb0 + kStep - 1) / kStep : 0;

    // ---- issue the global loads of this wave's tile t (no waiting).  Tiles past the wave's last
    // one are "issued" too, so that the number of loads in flight is the same on every path and
    // the compiler's wait counts stay exact: all their lanes read the first bytes of the last tile
    // (16 cache lines, already resident) and nothing consumes them.
    auto issue = [&](KVTile& t, int ti) {
        const bool real = ti < nw;
        const int kb = kb0 + min(ti, nw - 1) * kStep;
        const int kl = real ? k_lane : 0, vl = real ? v_lane : 0;
        // the second page exists only if the request has tokens there
        int pg0 = bt[kb >> 4];
        int pg1 = (kb + kP < kv_total) ? bt[(kb >> 4) + 1] : pg0;
        pg0 = min(max(pg0, 0), a.n_pages - 1);
        pg1 = min(max(pg1, 0), a.n_pages - 1);
        const char* kp0 = k_head + (size_t)pg0 * page_bytes;
        const char* kp1 = k_head + (size_t)pg1 * page_bytes;
        const char* vp0 = v_head + (size_t)pg0 * page_bytes;
        const char* vp1 = v_head + (size_t)pg1 * page_bytes;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            t.k[0][kk] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const s16x8*>(kp0 + kl + 64 * kk));
            t.k[1][kk] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const s16x8*>(kp1 + kl + 64 * kk));
        }
        // V: lane copies 16-byte chunk li of keys 4 r + lg, r = 0..7 (r >= 4: second page)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            t.v[r] = *reinterpret_cast<const s16x8*>(vp0 + vl + 1024 * r);
            t.v[4 + r] = *reinterpret_cast<const s16x8*>(vp1 + vl + 1024 * r);
        }
    };

    // The K/V stream does not depend on Q: start it before anything else of the segment.
    KVTile ta, tb;
    if (nw > 0) {
        issue(ta, 0);
        issue(tb, 1);
    }

    // ---- Q^T operands: lane holds query row (mt*16 + li), d = 32 kk + 8 lg .. +7.  They are the
    // same for the 4 waves and for every tile, so they live in LDS ([mt*4 + kk][lane] x 16 bytes,
    // read back lane-contiguous) instead of 16 registers per query tile.
    char* qbuf = smem + kQOff;
    int lim[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int m = mt * 16 + li;
        lim[mt] = m < M_g ? c + j0 + m / G : -1;
    }
    for (int pr = w; pr < MT * 4; pr += kWaves) {
        const int mt = pr >> 2, kk = pr & 3;
        const int m = mt * 16 + li;
        const bool ok = m < M_g;
        const int j = j0 + m / G, gq = m % G;
        const uint16_t* qp = a.q + ((size_t)(q0 + (ok ? j : j0)) * a.H_q + kvh * G + (ok ? gq : 0)) * kD + 8 * lg + 32 * kk;
        s16x8 t = *reinterpret_cast<const s16x8*>(qp);
        if (!ok) t = s16x8{0, 0, 0, 0, 0, 0, 0, 0};
        *reinterpret_cast<s16x8*>(qbuf + (pr * 64 + lane) * 16) = t;
    }
    __syncthreads();

    FSR_STAMP(seg_no * 5 + 3);
    float m_run[MT], l_run[MT];
    f32x4 acc[MT][8];
    auto reset_state = [&]() {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            m_run[mt] = -INFINITY;
            l_run[mt] = 0.0f;
#pragma unroll
            for (int db = 0; db < 8; ++db) acc[mt][db] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
    };
    reset_state();

    // ---- phase 1 of a tile: V to LDS, S^T = K Q^T on the matrix cores; afterwards the tile's
    // registers are free for the next loads.
    // s[mt][kt][e] = score(key kb + 16 kt + 4 lg + e, query mt*16 + li)
    auto stage_and_scores = [&](KVTile& t, int kb, f32x4 (&s)[MT][2]) {
        if (kb + kTile > kv_total) {  // slots past the request's last token may hold anything: zero them
#pragma unroll
            for (int r = 0; r < 8; ++r)
                if (kb + 4 * r + lg >= kv_total) t.v[r] = s16x8{0, 0, 0, 0, 0, 0, 0, 0};
        }
#pragma unroll
        for (int r = 0; r < 8; ++r)
            *reinterpret_cast<s16x8*>(vbuf + ((r & 1) ? vw_odd : vw_even) + 1024 * r) = t.v[r];
        // all Q^T operands first (one batch of LDS reads in flight), then the matrix instructions
        bf16x8 qop[MT][4];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int kk = 0; kk < 4; ++kk)
                qop[mt][kk] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const s16x8*>(qbuf + ((mt * 4 + kk) * 64 + lane) * 16));
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            s[mt][0] = s[mt][1] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                s[mt][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(t.k[0][kk], qop[mt][kk], s[mt][0], 0, 0, 0);
                s[mt][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(t.k[1][kk], qop[mt][kk], s[mt][1], 0, 0, 0);
            }
        }
        __builtin_amdgcn_sched_group_barrier(0x200, 8, 0);       // V stores
        __builtin_amdgcn_sched_group_barrier(0x100, 4 * MT, 0);  // Q^T operand reads
        __builtin_amdgcn_sched_group_barrier(0x008, 8 * MT, 0);  // score MFMAs
    };

    // raw scores of all query tiles with the keys a row may not see set to -inf
    auto masked_scores = [&](int kb, const f32x4 (&s)[MT][2], float (&x)[MT][8]) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                for (int e = 0; e < 4; ++e) x[mt][kt * 4 + e] = s[mt][kt][e];
        if (kb + kTile > c + j0 + 1) {  // only the item's last keys are causal-masked or past the end
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (kb + 16 * kt + 4 * lg + e > lim[mt]) x[mt][kt * 4 + e] = -INFINITY;
        }
    };
    auto max8 = [](const float (&x)[8]) {
        return fmaxf(fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3])), fmaxf(fmaxf(x[4], x[5]), fmaxf(x[6], x[7])));
    };
    // V^T operands of the 8 d-blocks from the LDS tile: element e < 4 is key 4 lg + e of the tile's
    // first 16 keys, e >= 4 is key 16 + 4 lg + (e - 4) -- the order in which S^T's accumulators
    // hold the keys
    auto load_vops = [&](bf16x8 (&vop)[8]) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
        for (int db = 0; db < 8; ++db) {
            const s16x4 t0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(vbuf + vr_off[db]));
            const s16x4 t1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(vbuf + vr_off[db] + 16 * 256));
            vop[db] = __builtin_bit_cast(bf16x8, s16x8{t0[0], t0[1], t0[2], t0[3], t1[0], t1[1], t1[2], t1[3]});
        }
    };
    // probabilities of query tile mt against reference m_run[mt], as a bf16 hi + lo pair
    // (hi = truncation, lo = rounded remainder), then O^T += V^T P^T on the matrix cores.
    // The softmax scale (times log2 e) is folded into the exponent.
    auto probs_and_pv = [&](const float (&x)[8], int mt, const bf16x8 (&vop)[8]) {
        const float neg_m = m_run[mt] == -INFINITY ? 0.0f : -m_run[mt];
        float psum = 0.0f;
        uint32_t hi_pk[4];
        bf16x8 pl;
#pragma unroll
        for (int e = 0; e < 8; e += 2) {
            const float p0 = fast_exp2(fmaf(x[e], a.scale_log2, neg_m)), p1 = fast_exp2(fmaf(x[e + 1], a.scale_log2, neg_m));
            psum += p0 + p1;
            const uint32_t b0 = __builtin_bit_cast(uint32_t, p0), b1 = __builtin_bit_cast(uint32_t, p1);
            hi_pk[e >> 1] = __builtin_amdgcn_perm(b1, b0, 0x07060302u);
            pl[e] = (__bf16)(p0 - __builtin_bit_cast(float, b0 & 0xffff0000u));
            pl[e + 1] = (__bf16)(p1 - __builtin_bit_cast(float, b1 & 0xffff0000u));
        }
        l_run[mt] += psum;
        const bf16x8 ph = __builtin_bit_cast(bf16x8, u32x4{hi_pk[0], hi_pk[1], hi_pk[2], hi_pk[3]});
#pragma unroll
        for (int db = 0; db < 8; ++db) {
            acc[mt][db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vop[db], ph, acc[mt][db], 0, 0, 0);
            acc[mt][db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vop[db], pl, acc[mt][db], 0, 0, 0);
        }
    };
    auto end_of_tile = [&]() {  // the next tile's V stores must not overtake this tile's transposed reads
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    };

    // ---- FAST LOOP.  A row's exponent reference m_run is fixed at the row maximum of the first tile
    // in which the row sees a key and is then left alone: later probabilities may exceed 1, which
    // fp32 absorbs (they stay below 2^kFastSlack, and O / l does not depend on the reference), so no
    // instruction but the matrix cores' touches the accumulators and no lane talks to another.
    // If a later score does exceed the reference by more than kFastSlack the wave gives the fast
    // loop up and redoes its tiles with the exact, rescaling loop below.
    // Two tiles are in flight per wave (ping-pong buffers, 32 KB), so a wave's progress is set by
    // its fair share of HBM bandwidth and not by load latency plus its own arithmetic.
    constexpr float kFastSlack = 64.0f;
    bool lane_ok = true;
    auto fast_softmax_pv = [&](int kb, const f32x4 (&s)[MT][2]) {
        bf16x8 vop[8];
        load_vops(vop);
        float x[MT][8], lane_max[MT];
        masked_scores(kb, s, x);
        bool any = false;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            lane_max[mt] = a.scale_log2 * max8(x[mt]);
            any |= lane_max[mt] > m_run[mt] + kFastSlack;
        }
        if (__builtin_amdgcn_ballot_w64(any) != 0) {  // first keys of a row, or trouble
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                float row_max = fmaxf(lane_max[mt], __shfl_xor(lane_max[mt], 16, 64));
                row_max = fmaxf(row_max, __shfl_xor(row_max, 32, 64));
                if (m_run[mt] == -INFINITY) m_run[mt] = row_max;
                else if (row_max > m_run[mt] + kFastSlack) lane_ok = false;
            }
        }
        // straight-line from here: the matrix instructions of one query tile overlap the
        // exponentials of the next
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) probs_and_pv(x[mt], mt, vop);
        end_of_tile();
    };
    bool redo = false;
    if (nw > 0) {
        f32x4 s[MT][2];
        for (int t = 0; t < nw; t += 2) {
            stage_and_scores(ta, kb0 + t * kStep, s);
            __builtin_amdgcn_sched_barrier(0);
            issue(ta, t + 2);
            __builtin_amdgcn_sched_barrier(0);
            if (seg_no == 0 && t < 24) FSR_STAMP(16 + 2 * t);
            fast_softmax_pv(kb0 + t * kStep, s);
            if (seg_no == 0 && t < 24) FSR_STAMP(17 + 2 * t);
            const bool second = t + 1 < nw;
            if (second) stage_and_scores(tb, kb0 + (t + 1) * kStep, s);
            __builtin_amdgcn_sched_barrier(0);
            issue(tb, t + 3);
            __builtin_amdgcn_sched_barrier(0);
            if (seg_no == 0 && t < 24) FSR_STAMP(18 + 2 * t);
            if (second) fast_softmax_pv(kb0 + (t + 1) * kStep, s);
            if (seg_no == 0 && t < 24) FSR_STAMP(19 + 2 * t);
        }
        redo = __builtin_amdgcn_ballot_w64(!lane_ok) != 0;
    }

    // ---- EXACT LOOP (fallback, one tile in flight).  The reference of a row is raised, and sums
    // and accumulators rescaled, whenever a score exceeds it by more than kSlack.  Loop shape: the
    // inner loop finishes the pending tile, then stages and scores the next one; it is left only
    // when that tile needs a higher reference, which the outer loop handles.
    if (redo) {
        constexpr float kSlack = 8.0f;
        reset_state();
        auto issue_one = [&](KVTile& t, int ti) {
            if (ti < nw) issue(t, ti);
        };
        auto needs_raise = [&](int kb, const f32x4 (&s)[MT][2]) {
            bool any = false;
            float x[MT][8];
            masked_scores(kb, s, x);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) any |= a.scale_log2 * max8(x[mt]) > m_run[mt] + kSlack;
            return __builtin_amdgcn_ballot_w64(any) != 0;
        };
        auto raise_refs = [&](int kb, const f32x4 (&s)[MT][2]) {
            float x[MT][8];
            masked_scores(kb, s, x);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                const float lane_max = a.scale_log2 * max8(x[mt]);
                float row_max = fmaxf(lane_max, __shfl_xor(lane_max, 16, 64));
                row_max = fmaxf(row_max, __shfl_xor(row_max, 32, 64));
                const float m_new = row_max > m_run[mt] + kSlack ? row_max : m_run[mt];
                const float alpha = m_new == -INFINITY ? 1.0f : fast_exp2(m_run[mt] - m_new);
                m_run[mt] = m_new;
                l_run[mt] *= alpha;
#pragma unroll
                for (int db = 0; db < 8; ++db) acc[mt][db] *= alpha;
            }
        };
        auto exact_softmax_pv = [&](int kb, const f32x4 (&s)[MT][2]) {
            bf16x8 vop[8];
            load_vops(vop);
            float x[MT][8];
            masked_scores(kb, s, x);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) probs_and_pv(x[mt], mt, vop);
            end_of_tile();
        };
        f32x4 s[MT][2];
        int t = 0;
        issue_one(ta, 0);
        stage_and_scores(ta, kb0, s);
        issue_one(ta, 1);
        bool more = true;
        while (more) {
            raise_refs(kb0 + t * kStep, s);
            for (;;) {
                exact_softmax_pv(kb0 + t * kStep, s);
                if (++t >= nw) {
                    more = false;
                    break;
                }
                stage_and_scores(ta, kb0 + t * kStep, s);
                issue_one(ta, t + 1);
                if (needs_raise(kb0 + t * kStep, s)) break;
            }
        }
    }

    FSR_STAMP(seg_no * 5 + 4);
    // ---- row sums live spread over the 4 lane groups
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        l_run[mt] += __shfl_xor(l_run[mt], 16, 64);
        l_run[mt] += __shfl_xor(l_run[mt], 32, 64);
    }

    // ---- merge the 4 waves (each saw a disjoint set of keys)
    float* red_m = reinterpret_cast<float*>(smem + kMlOff);   // [kWaves][96]
    float* red_l = red_m + kWaves * 16 * kMaxMT;
    float* red_o = reinterpret_cast<float*>(smem);            // [kWaves][16][kRedStride], shares the V tiles' space
    __syncthreads();
    if (lg == 0) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            red_m[w * 16 * kMaxMT + mt * 16 + li] = m_run[mt];
            red_l[w * 16 * kMaxMT + mt * 16 + li] = l_run[mt];
        }
    }
    __syncthreads();
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
                float ms = -INFINITY;
#pragma unroll
                for (int ww = 0; ww < kWaves; ++ww) ms = fmaxf(ms, red_m[ww * 16 * kMaxMT + m]);
                const float mu = ms == -INFINITY ? 0.0f : ms;
                float ls = 0.0f;
#pragma unroll
                for (int ww = 0; ww < kWaves; ++ww)
                    ls += red_l[ww * 16 * kMaxMT + m] * fast_exp2(red_m[ww * 16 * kMaxMT + m] - mu);
                if (final_out) {
                    const int j = j0 + m / G, h = kvh * G + m % G;
                    const size_t o_idx = ((size_t)(q0 + j) * a.H_q + h) * kD + d0;
                    const float inv = 1.0f / ls;
                    s0 *= inv;
                    s1 *= inv;
                    if (a.out_bf16) {
                        s16x8 pk;
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            pk[e] = (short)f32_to_bf16_rne(s0[e]);
                            pk[4 + e] = (short)f32_to_bf16_rne(s1[e]);
                        }
                        *reinterpret_cast<s16x8*>(reinterpret_cast<uint16_t*>(a.out) + o_idx) = pk;
                    } else {
                        float* dst = reinterpret_cast<float*>(a.out) + o_idx;
                        *reinterpret_cast<f32x4*>(dst) = s0;
                        *reinterpret_cast<f32x4*>(dst + 4) = s1;
                    }
                    if (a.lse && d0 == 0) a.lse[(size_t)(q0 + j) * a.H_q + h] = (ms + __log2f(ls)) * kLn2;
                } else {
                    float* dst = a.part_o + ((size_t)slot * a.m_cap + m) * kD + d0;
                    *reinterpret_cast<f32x4*>(dst) = s0;
                    *reinterpret_cast<f32x4*>(dst + 4) = s1;
                    if (d0 == 0) {
                        float* ml = a.part_ml + ((size_t)slot * a.m_cap + m) * 2;
                        ml[0] = ms;
                        ml[1] = ls;
                    }
                }
            }
        }
        __syncthreads();
    }
}

template <int MTMAX>
__device__ __forceinline__ void attend_dispatch(const FastArgs& a, int mt, int i, int kvh, int c, int q0, int q_len,
                                                int j0, int rows_g, int tile_a, int tile_e, bool final_out, int slot,
                                                char* smem, int seg_no = 0) {
#define FSR_SEG(MT) attend_segment<MT>(a, i, kvh, c, q0, q_len, j0, rows_g, tile_a, tile_e, final_out, slot, smem, seg_no)
    if constexpr (MTMAX == 1) {
        FSR_SEG(1);
    } else if constexpr (MTMAX == 2) {
        if (mt == 1) FSR_SEG(1); else FSR_SEG(2);
    } else if constexpr (MTMAX == 3) {
        if (mt == 1) FSR_SEG(1); else if (mt == 2) FSR_SEG(2); else FSR_SEG(3);
    } else if constexpr (MTMAX == 4) {
        if (mt <= 2) FSR_SEG(2); else if (mt == 3) FSR_SEG(3); else FSR_SEG(4);
    } else {
        if (mt <= 2) FSR_SEG(2); else if (mt <= 4) FSR_SEG(4); else FSR_SEG(6);
    }
#undef FSR_SEG
}

// Persistent grid: nb workgroups of 256 threads; workgroup b takes flattened tiles
// [b T / nb', (b+1) T / nb') with nb' = min(nb, T).
template <int MTMAX>
__global__ __launch_bounds__(kThreads) void attn_stream_kernel(FastArgs a) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    int* pref = reinterpret_cast<int*>(smem + kPrefOff);
    FSR_STAMP(0);
#ifdef FSR_TIMING
    if (threadIdx.x == 0) a.dbg[(size_t)blockIdx.x * 512 + 126 * 4] = clock64();
#endif
    build_tile_prefix(a, pref, reinterpret_cast<int*>(smem + kScanOff));
    FSR_STAMP(1);
    const long long T = (long long)pref[a.B] * a.H_kv;
    const int nb = (int)min((long long)a.nb, T);
    const int b = blockIdx.x;
    if (b >= nb) return;
    long long t = (long long)b * T / nb;
    const long long t1 = (long long)(b + 1) * T / nb;
    int seg_no = 0;
    while (t < t1) {
        const Item it = locate(pref, a.B, a.H_kv, t);
        const int tile_e = (int)min((long long)it.nt, it.tile + (t1 - t));
        const int q0 = a.cu_q[it.i], q_len = a.cu_q[it.i + 1] - q0;
        const int c = max(a.ctx[it.i], 0);
        const int rows = a.G * q_len;
        if (rows <= 16 * MTMAX) {
            const bool whole = it.tile == 0 && tile_e == it.nt;
            const int slot = b * 2 + (it.tile > 0 ? 0 : 1);
            attend_dispatch<MTMAX>(a, (rows + 15) >> 4, it.i, it.g, c, q0, q_len, 0, q_len, it.tile, tile_e, whole, slot, smem, min(seg_no, 2));
            ++seg_no;
        } else if (it.tile == 0) {
            // more rows than a partial slot holds: the workgroup owning the item's first tile does
            // the whole item, in passes over groups of rows; the other workgroups skip it
            const int rows_per_pass = (16 * MTMAX) / a.G;
            for (int j0 = 0; j0 < q_len; j0 += rows_per_pass) {
                const int rows_g = min(rows_per_pass, q_len - j0);
                attend_dispatch<MTMAX>(a, (a.G * rows_g + 15) >> 4, it.i, it.g, c, q0, q_len, j0, rows_g, 0, it.nt, true, 0, smem);
            }
        }
        t += tile_e - it.tile;
    }
    FSR_STAMP(15);
#ifdef FSR_TIMING
    if (threadIdx.x == 0) a.dbg[(size_t)blockIdx.x * 512 + 127 * 4] = clock64();
#endif
}

// Combine the partials of items cut by share boundaries.  grid = nb.  Workgroup b is
// responsible for the item that contains its first tile if that item starts inside the
// previous workgroup's share; the pieces are then slot 1 of b-1 and slot 0 of b, b+1, ...
// while their shares start inside the item.
__global__ __launch_bounds__(kThreads) void attn_fixup_kernel(FastArgs a) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    int* pref = reinterpret_cast<int*>(smem + kPrefOff);
    build_tile_prefix(a, pref, reinterpret_cast<int*>(smem + kScanOff));
    const long long T = (long long)pref[a.B] * a.H_kv;
    const int nb = (int)min((long long)a.nb, T);
    const int b = blockIdx.x;
    if (b == 0 || b >= nb) return;
    const long long t0 = (long long)b * T / nb;
    const Item it = locate(pref, a.B, a.H_kv, t0);
    if (it.tile == 0) return;                       // the boundary falls between two items
    const long long item_start = t0 - it.tile, item_end = item_start + it.nt;
    if (item_start < (long long)(b - 1) * T / nb) return;  // an earlier workgroup is responsible
    const int q0 = a.cu_q[it.i], q_len = a.cu_q[it.i + 1] - q0;
    const int M = a.G * q_len;
    if (M > a.m_cap) return;                        // such items are never cut
    int b_last = b;
    while (b_last + 1 < nb && (long long)(b_last + 1) * T / nb < item_end) ++b_last;
    for (int e = threadIdx.x; e < M * (kD / 4); e += kThreads) {
        const int m = e / (kD / 4), d0 = (e % (kD / 4)) * 4;
        float m_star = -INFINITY;
        for (int bb = b - 1; bb <= b_last; ++bb) {
            const int slot = bb * 2 + (bb == b - 1 ? 1 : 0);
            m_star = fmaxf(m_star, a.part_ml[((size_t)slot * a.m_cap + m) * 2]);
        }
        const float mu = m_star == -INFINITY ? 0.0f : m_star;
        f32x4 o = f32x4{0.f, 0.f, 0.f, 0.f};
        float l = 0.0f;
        for (int bb = b - 1; bb <= b_last; ++bb) {
            const int slot = bb * 2 + (bb == b - 1 ? 1 : 0);
            const float* ml = a.part_ml + ((size_t)slot * a.m_cap + m) * 2;
            const float wgt = fast_exp2(ml[0] - mu);
            l += ml[1] * wgt;
            o += *reinterpret_cast<const f32x4*>(a.part_o + ((size_t)slot * a.m_cap + m) * kD + d0) * wgt;
        }
        o *= 1.0f / l;
        const int j = m / a.G, h = it.g * a.G + m % a.G;
        const size_t o_idx = ((size_t)(q0 + j) * a.H_q + h) * kD + d0;
        if (a.out_bf16) {
            ushort4 pk;
            pk.x = f32_to_bf16_rne(o[0]);
            pk.y = f32_to_bf16_rne(o[1]);
            pk.z = f32_to_bf16_rne(o[2]);
            pk.w = f32_to_bf16_rne(o[3]);
            *reinterpret_cast<ushort4*>(reinterpret_cast<uint16_t*>(a.out) + o_idx) = pk;
        } else {
            *reinterpret_cast<f32x4*>(reinterpret_cast<float*>(a.out) + o_idx) = o;
        }
        if (a.lse && d0 == 0) a.lse[(size_t)(q0 + j) * a.H_q + h] = (m_star + __log2f(l)) * kLn2;
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
    // the block table is read-only input: reading it through the constant address space lets the
    // compiler use scalar loads for the (wave-uniform) page look-ups
    const const_i32* bt = (const const_i32*)(a.bt + (size_t)i * a.max_pages);
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
    int nb;      // workgroups of the persistent grid
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
    if ((long long)p->max_pages * p->P > (1LL << 30)) return fail(FSR_EUNSUP, "%s: max_pages * P exceeds 2^30 tokens", who);
    return FSR_OK;
}

// Workgroups of the persistent grid: one per compute unit of the current device.
int persistent_blocks() {
    static thread_local int cached_dev = -1, cached_cus = 0;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) {
        (void)hipGetLastError();
        return 256;  // no device visible (host-only size query): MI355X has 256 compute units
    }
    if (dev != cached_dev) {
        int cus = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) {
            (void)hipGetLastError();
            cus = 256;
        }
        cached_dev = dev;
        cached_cus = cus;
    }
    return cached_cus;
}

Plan make_plan(const fsr_attn_params& p) {
    Plan pl{};
    const int G = p.H_q / p.H_kv;
    pl.fast = p.dtype == FSR_BF16 && p.D == kD && p.P == kP && G <= 16 && p.B <= kMaxB;
    if (!pl.fast) return pl;
    // rows of one request that share a KV head: G * max_q_len (unknown bound -> the widest kernel)
    const long long m_rows = p.max_q_len > 0 ? (long long)G * p.max_q_len : 16 * kMaxMT;
    const int mt = (int)std::min<long long>((m_rows + 15) / 16, kMaxMT);
    pl.mt_max = mt <= 4 ? mt : kMaxMT;
    // the workspace is sized for up to 1024 workgroups so that its size does not depend on the device
    pl.nb = std::min(persistent_blocks(), 1024);
    pl.bytes_o = align_up((size_t)1024 * 2 * 16 * pl.mt_max * kD * sizeof(float), 256);
    pl.bytes_ml = align_up((size_t)1024 * 2 * 16 * pl.mt_max * 2 * sizeof(float), 256);
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
        a.out = out; a.lse = lse;
        a.part_o = (float*)workspace;
        a.part_ml = (float*)((char*)workspace + pl.bytes_o);
        a.B = p->B; a.H_q = p->H_q; a.H_kv = p->H_kv; a.G = p->H_q / p->H_kv;
        a.max_pages = p->max_pages; a.n_pages = p->n_pages;
        a.nb = pl.nb; a.m_cap = 16 * pl.mt_max; a.out_bf16 = p->out_dtype == FSR_BF16;
        a.scale_log2 = p->scale * kLog2e;
#ifdef FSR_TIMING
        a.dbg = (long long*)((char*)workspace + need);  // the timing build expects 1 MiB of slack after the workspace
#endif
        const dim3 grid(pl.nb), block(kThreads);
        switch (pl.mt_max) {
            case 1: hipLaunchKernelGGL(attn_stream_kernel<1>, grid, block, kFastSmem, s, a); break;
            case 2: hipLaunchKernelGGL(attn_stream_kernel<2>, grid, block, kFastSmem, s, a); break;
            case 3: hipLaunchKernelGGL(attn_stream_kernel<3>, grid, block, kFastSmem, s, a); break;
            case 4: hipLaunchKernelGGL(attn_stream_kernel<4>, grid, block, kFastSmem, s, a); break;
            default: hipLaunchKernelGGL(attn_stream_kernel<6>, grid, block, kFastSmem, s, a); break;
        }
        if ((rc = check_launch("attn_stream_kernel")) != FSR_OK) return rc;
        hipLaunchKernelGGL(attn_fixup_kernel, grid, block, kFastSmem, s, a);
        return check_launch("attn_fixup_kernel");
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
