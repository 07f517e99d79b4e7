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
//   * each of the 4 waves streams its own tiles with a two-tile register prefetch, every load
//     taking 1 KB of consecutive bytes (four whole key rows) with the non-temporal hint: K and V
//     are staged through wave-private, XOR-swizzled LDS tiles; K is read back in the A-operand
//     layout of v_mfma_f32_16x16x32_bf16 (S^T = K Q^T), V transposed with ds_read_b64_tr_b16
//     (O^T = V^T P^T);
//   * a request whose rows per KV head exceed four query tiles is taken by two teams of two
//     waves in one pass over its keys (see attend_segment), so that its K/V bytes still come
//     from HBM once;
//   * S^T's accumulator layout is exactly the B-operand layout P^T needs, so the softmax
//     runs in registers with two cross-lane steps per row;
//   * P is fed to the matrix cores as a bf16 hi + lo pair: the result is accurate to fp32
//     rounding instead of bf16 rounding of the probabilities;
//   * an item that lies inside one share is normalised and written directly; an item cut by
//     a share boundary leaves (reference, sum, accumulator) partials -- at most two per workgroup
//     -- and the workgroup whose piece arrives last combines them, in the same launch.
// Generic path (fp32 or bf16, D in {64,128}, any page size): one wave per (row, head), plain
// fp32 FMAs -- a correctness path for small or unusual shapes, not a bandwidth kernel.
#include <algorithm>
#include <atomic>
#include <map>
#include <mutex>
#include <type_traits>

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
// K/V bytes are addressed through the global address space explicitly: a pointer rebuilt from scalar
// halves is otherwise a generic one, and its loads are "flat" ones that also count as LDS accesses
typedef const __attribute__((address_space(1))) char gmem_char;
typedef const __attribute__((address_space(1))) __attribute__((__vector_size__(8 * sizeof(short)))) short gmem_s16x8;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;

constexpr int kD = 128;           // head dim of the fast path
constexpr int kP = 16;            // page size of the fast path
constexpr int kTile = 32;         // keys per wave tile
constexpr int kWaves = 4;
constexpr int kThreads = kWaves * 64;
constexpr int kMaxMT = 4;         // up to 64 query rows (G * suffix positions) per row group
constexpr int kMaxB = 4096;       // requests whose tile prefix fits the LDS table
constexpr int kRedStride = kD + 4;  // padded row of the wave-merge buffer (floats)
// LDS map, fixed part: [V tiles of the 4 waves | wave-merge buffer] (shared region), wave maxima and
// sums, Q^T operands.  The merge buffer holds the accumulators of RT query tiles of all 4 waves at a
// time: merging a segment's query tiles in one batch costs two workgroup barriers instead of two per
// tile (what a merge costs is mostly LDS traffic, though: about 0.8 us per query tile either way).
constexpr int kVTileBytes = kTile * kD * 2;
constexpr int kRedBytes = kWaves * 16 * kRedStride * 4;
constexpr int kMlBytes = 2 * kWaves * 16 * kMaxMT * 4;
constexpr int kQBytes = kMaxMT * 4 * 64 * 16;
constexpr int kWideMT = 3;  // query tiles per team of a two-team segment (see attend_segment)
constexpr int kQTeamBytes = kWideMT * 4 * 64 * 16;
template <int RT, bool WIDE>
struct Lds {
    // a wave's own region: its K and V tiles while it streams, its accumulators (RT query tiles) when it merges
    static constexpr int kWaveRegion = 2 * kVTileBytes > RT * (kRedBytes / kWaves) ? 2 * kVTileBytes : RT * (kRedBytes / kWaves);
    static constexpr int kStage = kWaves * kWaveRegion;
    static constexpr int kMl = kStage;
    static constexpr int kQ = kMl + kMlBytes;  // Q^T operands of the current item: [query tile * 4][64 lanes][16 B], per team
    static constexpr int kFixed = kQ + (WIDE ? 2 * kQTeamBytes : kQBytes);
};
// The kernel that reads a plan has the LDS to itself and merges all query tiles of a segment at once.  The
// kernel that builds its own schedule keeps three tables sized from the call's B behind the fixed part --
// weighted tile prefix (64-bit, B + 1 entries), scan scratch, and copies of the row offsets and context
// lengths the prefix has loaded anyway (the walker reads them there) -- and merges two tiles at a time,
// which still fits 160 KB at B = 4096.
constexpr int kStreamRT = 2;
__host__ __device__ constexpr int stream_fixed_smem(bool wide) { return wide ? Lds<kStreamRT, true>::kFixed : Lds<kStreamRT, false>::kFixed; }
__host__ __device__ constexpr int planned_smem(int mt_max, bool wide) {
    return wide ? Lds<kWideMT, true>::kFixed
                : mt_max <= 1 ? Lds<1, false>::kFixed : mt_max == 2 ? Lds<2, false>::kFixed : mt_max == 3 ? Lds<3, false>::kFixed : Lds<4, false>::kFixed;
}
// the schedule tables, as offsets from where they start
__host__ __device__ constexpr int scan_off(int B) { return ((B + 1) * 8 + 15) / 16 * 16; }
__host__ __device__ constexpr int cu_off(int B) { return scan_off(B) + 64; }
__host__ __device__ constexpr int ctx_off(int B) { return cu_off(B) + (B + 4) * 4; }
__host__ __device__ constexpr int tables_bytes(int B) { return ctx_off(B) + (B + 4) * 4; }
// Measured: a tile takes 2.0 / 2.4 / 2.5 us per wave with 1 / 2 / 3 query tiles riding on it (bandwidth, not the
// matrix work, sets the pace), and taking up an item costs a workgroup 6 to 10 us of merge, count and refill.
// Swept on four batches of the 16-request shape and on the 128- and 512-request shapes: base 3..6 with 12..20
// phantom tiles is a plateau, 5 to 9 % under base 1 with 8.
// With many items per workgroup the per-item costs average out and time follows the bytes, i.e. the tile count:
// the 256- and 512-request shapes keep gaining up to base 16 (another 8 % and 5 %), while the 16-request shape,
// where a workgroup holds one or two long items whose fixed costs grow with the query tiles, is best at 4.  The
// host therefore sets the base to twice the items per workgroup, between kCostBase and kCostBaseMax.
constexpr int kCostBase = 4;   // a tile costs cost_base + (16-row query tiles riding on it)
constexpr int kCostBaseMax = 16;
constexpr int kSegTiles = 16;  // what starting an item costs a workgroup (merge, refill), in tiles of that item
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
    float* part_o;   // [shares * 2, m_cap, D]   unnormalised accumulators of cut items
    float* part_ml;  // [shares * 2, m_cap, 4]   (exponent reference in log2 units, sum, call tag, unused)
    unsigned long long* arrivals;  // [shares + 1] (call id << 16 | pieces of a cut item that have arrived)
    unsigned long long call_id;    // distinguishes this call's counts and partials from whatever the workspace held before
    const int32_t* plan;           // schedule written by attn_plan_kernel (planned kernel only)
    uint32_t plan_key;             // what the plan must have been built for (planned kernel only)
    int B, H_q, H_kv, G, max_pages, n_pages;
    int nb;          // workgroups of the persistent grid
    int m_cap;       // rows (G * positions of a row group) a partial slot holds
    int wide;        // row groups hold two teams' worth of suffix positions (see attend_segment)
    int out_bf16;
    float scale_log2;
    const float* k_scale;  // 8-bit caches: per KV head, cached key = decode(byte) * k_scale[head]; else unused
    const float* v_scale;  // the same for values
    int cost_base;   // fixed part of a tile's cost (see tile_cost)
    int seg_tiles;   // phantom tiles in front of every item on the cost line (see the schedule)
};

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
// Stores that go to the device's point of coherence (past the per-die L2), for the few KB that
// workgroups hand to each other inside one launch: 16-byte buffer stores with the device-scope bit, so a
// wave's store instruction covers whole cache lines (narrower ones reach memory as partial-line writes).
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4_t;
constexpr int kStoreDeviceScope = 16;  // cache-policy bit "sc1" of the buffer store
__device__ __forceinline__ __amdgpu_buffer_rsrc_t partial_buffer(float* base) {
    return __builtin_amdgcn_make_buffer_rsrc(base, 0, 0x7fffffff, 0x00020000);
}
__device__ __forceinline__ void coherent_store4(__amdgpu_buffer_rsrc_t buf, size_t float_index, f32x4 v) {
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4_t, v), buf, (int)(float_index * 4), 0, kStoreDeviceScope);
}
__device__ __forceinline__ uint16_t f32_to_bf16_rne(float x) { return __builtin_bit_cast(uint16_t, (__bf16)x); }

// Swizzled byte offset of 16-byte chunk `ch` (0..15) of key row `key` in a [32][128] bf16 tile.
__device__ __forceinline__ int vtile_off(int key, int ch) { return key * 256 + ((ch ^ ((key & 7) << 1)) << 4); }

// ---------------------------------------------------------------------------------------
// Schedule.  An item is (request i, KV head g, row group k): the rows of request i that share KV
// head g, in groups of at most 16 * mt_max rows (whole suffix positions: rows_per_group = 16 *
// mt_max / G positions), so that a group's accumulators fit the kernel's registers.  Nearly always
// a request is one group.  Work is measured in cost units: a 32-key tile of a group costs
// cost_base + (16-row query tiles riding on it), so that shares of equal cost take about equal
// time whether a request has one suffix row or nine.  In front of its real tiles every item carries
// seg_tiles phantom tiles: they stand for what it costs a workgroup to take up an item at all
// (merging its waves, refilling the load pipeline), so a workgroup whose share spans an item
// boundary is handed fewer real tiles than one that streams a single item throughout.
// pref[i] = cost of the items of requests 0..i-1 for one KV head; on the flattened cost line the
// request's items follow each other head by head, and inside a head group by group.
// ---------------------------------------------------------------------------------------
struct Group {
    int j0, rows_g;  // suffix positions j0 .. j0 + rows_g - 1 of the request
    int nt, cost;    // tiles (phantom ones included) and cost of one tile
};

// Group of request (context c, q_len rows) that starts at suffix position j0.
// Suffix positions whose G * positions query rows fit mt_max query tiles: what one team of waves takes.
__device__ __forceinline__ int rows_per_team(const FastArgs& a, int mt_max) { return max((16 * mt_max) / a.G, 1); }
__device__ __forceinline__ int rows_per_group(const FastArgs& a, int mt_max) { return rows_per_team(a, mt_max) * (a.wide ? 2 : 1); }
__device__ __forceinline__ Group group_at(const FastArgs& a, int mt_max, int c, int q_len, int j0) {
    const int per_team = rows_per_team(a, mt_max);
    Group gr;
    gr.j0 = j0;
    gr.rows_g = min(rows_per_group(a, mt_max), q_len - j0);
    const int visible = min(c + j0 + gr.rows_g, a.max_pages * kP);  // keys the group's last row sees
    gr.nt = (visible + kTile - 1) / kTile + a.seg_tiles;
    const int rows_a = min(gr.rows_g, per_team), rows_b = gr.rows_g - rows_a;
    gr.cost = a.cost_base + min((a.G * rows_a + 15) >> 4, mt_max) + ((a.G * rows_b + 15) >> 4);
    return gr;
}

// Returns the largest per-tile cost of any item.
__device__ int build_cost_prefix(const FastArgs& a, int mt_max, long long* pref, long long* scratch, int* lds_cu, int* lds_ctx) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    long long carry = 0;
    int cmax = 1;
    for (int base = 0; base < a.B; base += kThreads) {
        const int i = base + threadIdx.x;
        long long units = 0;
        if (i < a.B) {
            const int cu0 = a.cu_q[i], cu1 = a.cu_q[i + 1], c = max(a.ctx[i], 0);
            const int ql = cu1 - cu0;
            if (i == 0) lds_cu[0] = cu0;
            lds_cu[i + 1] = cu1;
            lds_ctx[i] = c;
            for (int j0 = 0; j0 < ql; j0 += rows_per_group(a, mt_max)) {
                const Group gr = group_at(a, mt_max, c, ql, j0);
                units += (long long)gr.nt * gr.cost;
                cmax = max(cmax, gr.cost);
            }
        }
        const long long inc = wave_inclusive_scan(units);
        if (lane == 63) scratch[w] = inc;
        __syncthreads();
        long long before = 0, total = 0;
#pragma unroll
        for (int k = 0; k < kWaves; ++k) {
            if (k < w) before += scratch[k];
            total += scratch[k];
        }
        if (i < a.B) pref[i] = carry + before + inc - units;
        carry += total;
        __syncthreads();
    }
    if (threadIdx.x == 0) pref[a.B] = carry;
    cmax = wave_max_i(cmax);
    if (lane == 0) scratch[w] = cmax;
    __syncthreads();
    cmax = (int)max(max(scratch[0], scratch[1]), max(scratch[2], scratch[3]));
    __syncthreads();
    return cmax;
}

// Quotient of two non-negative numbers; nearly always both fit 32 bits, where the division is an
// order of magnitude cheaper than the 64-bit one.
__device__ __forceinline__ long long div_u(long long n, long long d) {
    if ((((unsigned long long)n | (unsigned long long)d) >> 32) == 0) return (long long)((unsigned)n / (unsigned)d);
    return n / d;
}

// Request whose items hold cost position x: largest i with pref[i] * H_kv <= x.
__device__ __forceinline__ int locate_request(const long long* pref, int B, int H_kv, long long x) {
    int lo = 0, hi = B;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (pref[mid] * H_kv <= x) lo = mid; else hi = mid;
    }
    return lo;
}

struct KVTile {
    bf16x8 k[2][4];
    s16x8 v[8];
};
// The same tile of an 8-bit cache: a key row is 128 bytes.  k[page][c]: key li of the page, the 16
// bytes d = 64 c + 16 lg .. +15; v[r]: key 8 r + lane / 8 of the tile, the 16 bytes d = 16 (lane % 8) .. +15.
struct KVTile8 {
    u32x4 k[2][2];
    u32x4 v[4];
};
template <bool KV8> struct TileOf { typedef KVTile type; };
template <> struct TileOf<true> { typedef KVTile8 type; };
typedef const __attribute__((address_space(1))) u32x4 gmem_u32x4;

// 4 E4M3 bytes -> 4 bf16 (exact: 3 mantissa bits fit bf16's 7), as two packed pairs.
__device__ __forceinline__ void e4m3x4_to_bf16(uint32_t w, uint32_t& lo, uint32_t& hi) {
    typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2;
    const f32x2 a = __builtin_amdgcn_cvt_pk_f32_fp8((int)w, false), b = __builtin_amdgcn_cvt_pk_f32_fp8((int)w, true);
    // (elements to scalars before the bit casts: a bit cast of a vector-element expression was seen to read element 0)
    const float a0 = a[0], a1 = a[1], b0 = b[0], b1 = b[1];
    lo = __builtin_amdgcn_perm(__builtin_bit_cast(uint32_t, a1), __builtin_bit_cast(uint32_t, a0), 0x07060302u);
    hi = __builtin_amdgcn_perm(__builtin_bit_cast(uint32_t, b1), __builtin_bit_cast(uint32_t, b0), 0x07060302u);
}
// 16 E4M3 bytes -> 16 bf16 in two registers-of-8
__device__ __forceinline__ void e4m3x16_to_bf16(u32x4 w, u32x4& first8, u32x4& next8) {
    const uint32_t w0 = w[0], w1 = w[1], w2 = w[2], w3 = w[3];
    uint32_t a0, a1, a2, a3, b0, b1, b2, b3;
    e4m3x4_to_bf16(w0, a0, a1);
    e4m3x4_to_bf16(w1, a2, a3);
    e4m3x4_to_bf16(w2, b0, b1);
    e4m3x4_to_bf16(w3, b2, b3);
    first8 = u32x4{a0, a1, a2, a3};
    next8 = u32x4{b0, b1, b2, b3};
}

// What a workgroup processes between two merges: tiles [tile_a, tile_e) of item (i, kvh) for the
// query rows j0 .. j0 + rows_g - 1 of the request.  final_out: the tiles are the whole item, so
// the result is normalised and written to `out`; otherwise it goes to partial slot `slot`.
struct Segment {
    int i, kvh, c, q0, q_len, j0, rows_g, tile_a, tile_e, slot;
    bool final_out;
    // an item cut by share boundaries: its pieces are the shares b_first .. b_last
    bool cut;
    int b_first, b_last;
};

// One wave's view of a segment's K/V tiles: keys kb0 + t * (kWaves * kTile), t = 0 .. nw-1.
struct KVStream {
    const const_i32* bt;  // the request's block table, read through the constant address space so
                          // that the (wave-uniform) page look-ups are scalar loads
    bool rec_pages;  // the pages of the wave's first two tiles come from a plan record instead (lane l of
    int pgv;         // pgv = the record's entry l % 16, i.e. the page that holds key kbeg + 16 (l % 16))
    gmem_char* k_head;   // caches offset to the KV head
    gmem_char* v_head;
    int kb0, nw, kv_total, kend;
    int kbeg;  // first key of the segment (tile_a * kTile): what a wave without tiles of its own reads as filler
    int step;  // keys from one tile of the wave to its next: 32 x the waves that share the segment's keys
    // the wave's team: its suffix positions j0_t .. j0_t + rows_t - 1; per_team = positions of a full team
    int team, j0_t, rows_t, per_team;
};

// Values that are the same in every lane, moved to scalar registers: addresses built from them
// are scalar, and loads through them (the page look-ups) are scalar loads that never wait on the
// vector-memory queue.
__device__ __forceinline__ int uniform(int x) { return __builtin_amdgcn_readfirstlane(x); }
template <typename T>
__device__ __forceinline__ T* uniform(T* p) {
    const unsigned long long v = reinterpret_cast<unsigned long long>(p);
    const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)v), hi = __builtin_amdgcn_readfirstlane((unsigned)(v >> 32));
    return reinterpret_cast<T*>(((unsigned long long)hi << 32) | lo);
}
__device__ __forceinline__ long long uniform(long long x) {
    const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)x), hi = __builtin_amdgcn_readfirstlane((unsigned)((unsigned long long)x >> 32));
    return (long long)(((unsigned long long)hi << 32) | lo);
}
__device__ __forceinline__ gmem_char* uniform(gmem_char* p) {
    const unsigned long long v = (unsigned long long)p;
    const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)v), hi = __builtin_amdgcn_readfirstlane((unsigned)(v >> 32));
    return (gmem_char*)(((unsigned long long)hi << 32) | lo);
}
__device__ __forceinline__ const const_i32* uniform(const const_i32* p) {
    const unsigned long long v = (unsigned long long)p;
    const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)v), hi = __builtin_amdgcn_readfirstlane((unsigned)(v >> 32));
    return (const const_i32*)(((unsigned long long)hi << 32) | lo);
}

// Cache layouts.  TM = false: a page holds one [P, D] block per KV head (keys of a head 256 bytes
// apart, heads 4 KB apart).  TM = true: a page holds one [H_kv, D] block per token (keys of a head
// H_kv * 256 bytes apart, heads 256 bytes apart).  A template parameter, so that the first layout
// keeps every offset as an instruction immediate.
// KV8 = true: the caches hold one byte per element (OCP E4M3, see stage_and_scores) instead of bf16.
template <bool TM, bool KV8>
__device__ __forceinline__ int key_stride(const FastArgs& a) { return (TM ? a.H_kv * kD : kD) * (KV8 ? 1 : 2); }
template <bool TM, bool KV8>
__device__ __forceinline__ int head_stride() { return (TM ? kD : kP * kD) * (KV8 ? 1 : 2); }

// teams = 1: the 4 waves split the segment's keys.  teams = 2: waves 0, 1 take the first per_team
// positions of the row group and waves 2, 3 the rest; the two waves of a team split the keys.
template <bool TM, bool KV8>
__device__ __forceinline__ KVStream make_stream(const FastArgs& a, const Segment& sg, int per_team, int teams) {
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wpt = kWaves / teams, team = w / wpt, wk = w % wpt;
    KVStream st;
    st.bt = (const const_i32*)(a.bt + (size_t)__builtin_amdgcn_readfirstlane(sg.i) * a.max_pages);
    st.rec_pages = false;
    st.pgv = 0;
    const int kvh = __builtin_amdgcn_readfirstlane(sg.kvh);
    st.k_head = (gmem_char*)a.k + (size_t)kvh * head_stride<TM, KV8>();
    st.v_head = (gmem_char*)a.v + (size_t)kvh * head_stride<TM, KV8>();
    const int c = __builtin_amdgcn_readfirstlane(sg.c), q_len = __builtin_amdgcn_readfirstlane(sg.q_len);
    st.kv_total = min(c + q_len, a.max_pages * kP);  // tokens of this request in the cache
    const int kbeg = __builtin_amdgcn_readfirstlane(sg.tile_a) * kTile;
    const int j0 = __builtin_amdgcn_readfirstlane(sg.j0), rows_g = __builtin_amdgcn_readfirstlane(sg.rows_g);
    st.team = team;
    st.per_team = per_team;
    st.j0_t = j0 + team * per_team;
    st.rows_t = teams == 1 ? rows_g : team == 0 ? min(rows_g, per_team) : rows_g - per_team;
    // keys any row of the team may see
    st.kend = min(min(__builtin_amdgcn_readfirstlane(sg.tile_e) * kTile, c + st.j0_t + st.rows_t), st.kv_total);
    st.kbeg = kbeg;
    st.step = wpt * kTile;
    st.kb0 = kbeg + wk * kTile;
    st.nw = st.kb0 < st.kend ? (st.kend - st.kb0 + st.step - 1) / st.step : 0;
    return st;
}

// Shares and workgroups.  The hardware hands consecutive workgroups of a grid to the dies (XCDs) in
// turn, so workgroup w runs on die w % kDies.  Share ids are assigned die by die: the workgroups of
// one die hold consecutive shares, and the pieces of an item cut by share boundaries nearly always
// sit behind one L2 (only the seven boundaries between dies separate neighbours).  Nothing depends
// on the hardware keeping to that order: the exchange below is correct across dies as well.
constexpr int kDies = 8;
__device__ __forceinline__ int share_of_block(int w, int n) {  // w < n workgroups take part
    const int die = w % kDies, idx = w / kDies;
    // workgroups w' < n with w' % kDies < die
    const int full = n / kDies, extra = n % kDies;
    return die * full + min(die, extra) + idx;
}

// Walks a share [x, x1) of the cost line and hands out its segments in order.  UNI: the walker runs
// in all lanes of a wave alike (the attention kernel), so what it looks up is moved to scalar
// registers; the plan kernel walks a different share in every lane.
template <bool UNI>
struct ShareWalker {
    const long long* pref;
    const int* lds_cu;   // LDS copies of cu_q (B + 1 entries) and of max(ctx_lens, 0)
    const int* lds_ctx;
    long long x, x1, T, q;
    int nb, r, b, mt_max;

    static __device__ __forceinline__ int uni(int v) { return UNI ? uniform(v) : v; }
    // nb shares of q or q + 1 units (the first r are the longer ones)
    __device__ void set_shares(long long total, int n) {
        T = total; nb = n;
        q = div_u(total, n);
        r = (int)(total - q * n);
    }
    __device__ long long share_start(int bb) const { return bb * q + min(bb, r); }
    __device__ int owner_of(long long upto) const {  // largest bb with share_start(bb) < upto; upto >= 1
        const long long y = upto - 1, longer = (long long)r * (q + 1);
        const int bb = y < longer ? (int)div_u(y, q + 1) : r + (int)div_u(y - longer, q);
        return min(bb, nb - 1);
    }
    // Next segment of the share; false when the share is exhausted.
    __device__ bool next(const FastArgs& a, Segment& sg) {
        while (x < x1) {
            // scalar loads (constant address space, uniform index): they must not queue behind the K/V
            // tile loads that are in flight while the next segment is being looked up
            const int ri = uni(locate_request(pref, a.B, a.H_kv, x));
            const int q0 = uni(lds_cu[ri]), q_len = uni(lds_cu[ri + 1]) - q0, c = uni(lds_ctx[ri]);
            // the KV head, then the row group, that hold position x
            const long long per_head = pref[ri + 1] - pref[ri], req_base = pref[ri] * a.H_kv;
            const int g = (int)div_u(x - req_base, per_head);
            long long base = req_base + g * per_head;
            Group gr = group_at(a, mt_max, c, q_len, 0);
            while (x >= base + (long long)gr.nt * gr.cost && gr.j0 + gr.rows_g < q_len) {
                base += (long long)gr.nt * gr.cost;
                gr = group_at(a, mt_max, c, q_len, gr.j0 + gr.rows_g);
            }
            const long long iend = base + (long long)gr.nt * gr.cost;
            // tiles [xt_a, xt_e) of the item, phantom tiles included, are this share's
            const int xt_a = (int)div_u(x - base, gr.cost);
            const int xt_e = x1 >= iend ? gr.nt : (int)div_u(x1 - base, gr.cost);
            const int nt = gr.nt - a.seg_tiles, tile_a = max(xt_a - a.seg_tiles, 0), tile_e = max(xt_e - a.seg_tiles, 0);
            x = x1 >= iend ? iend : x1;
            if (tile_e > tile_a) {
                sg.i = ri; sg.kvh = uni(g); sg.c = c; sg.q0 = q0; sg.q_len = q_len;
                sg.j0 = gr.j0; sg.rows_g = gr.rows_g; sg.tile_a = tile_a; sg.tile_e = tile_e;
                sg.final_out = tile_a == 0 && tile_e == nt;
                sg.slot = b * 2 + (tile_a > 0 ? 0 : 1);
                sg.cut = !sg.final_out;
                sg.b_first = sg.b_last = b;
                if (sg.cut) {
                    // pieces of this item: the shares that own its first .. last tile; share bb owns
                    // tile k iff share_start(bb) < base + (k + 1) * cost <= share_start(bb + 1)
                    sg.b_first = owner_of(base + (long long)(a.seg_tiles + 1) * gr.cost);
                    sg.b_last = owner_of(iend);
                }
                return true;
            }
        }
        return false;
    }
};

// Issue the global loads of the wave's tile ti (no waiting); bt = the table in which the tile's pages
// are looked up.  Tiles past the wave's last one are "issued" too, so that the number of loads in
// flight is the same on every path and the compiler's wait counts stay exact: all their lanes read
// the first bytes of the last tile (16 cache lines, already resident) and nothing consumes them; a
// wave that has no tile of the segment reads the first bytes of the segment's first tile.
// NT: the loads carry the non-temporal hint.  A tile is read once per launch, and reads that do not claim
// cache space draw 10 % more from HBM (measured on long uniform items: 5.9 -> 6.5 TB/s); segments whose two
// teams of waves read the same tile count on the second read hitting the cache and keep the ordinary loads.
template <bool NT, typename T>
__device__ __forceinline__ T tile_load(const T* p) {
    if constexpr (NT) return __builtin_nontemporal_load(p);
    else return *p;
}
// KL: K is loaded in the same pattern as V (see stage_and_scores).
template <bool TM, bool KV8, bool FIRST = false, bool NT = false, bool KL = false>
__device__ __forceinline__ void issue_tile(const FastArgs& a, const KVStream& sv, typename TileOf<KV8>::type& t, int ti) {
    const int lane = threadIdx.x & 63, lg = lane >> 4, li = lane & 15;
    KVStream st;
    st.bt = uniform(sv.bt); st.k_head = uniform(sv.k_head); st.v_head = uniform(sv.v_head);
    st.kb0 = uniform(sv.kb0); st.nw = uniform(sv.nw); st.kv_total = uniform(sv.kv_total); st.kbeg = uniform(sv.kbeg);
    st.step = uniform(sv.step);
    ti = uniform(ti);
    const bool real = ti < st.nw;
    const int kb = st.nw > 0 ? st.kb0 + min(ti, st.nw - 1) * st.step : st.kbeg;
    // per-lane byte offsets inside a (page, head) block: every load is then
    // "uniform base + this offset + immediate", with no per-load address arithmetic
    const int ks = key_stride<TM, KV8>(a);
    const size_t page_bytes = (size_t)a.H_kv * kP * kD * (KV8 ? 1 : 2);
    int pg0, pg1;
    if (FIRST && sv.rec_pages) {
        // from the plan record (already clamped to the pool and to the request's last page): no look-up
        // stands between reading the record and sending for the tiles
        const int idx = uniform((kb - st.kbeg) >> 4);  // at most 2 * 3 + 8 = 14
        pg0 = __builtin_amdgcn_readlane(sv.pgv, idx);
        pg1 = __builtin_amdgcn_readlane(sv.pgv, idx + 1);
    } else {
        // the second page exists only if the request has tokens there
        pg0 = st.bt[kb >> 4];
        pg1 = (kb + kP < st.kv_total) ? st.bt[(kb >> 4) + 1] : pg0;
        pg0 = min(max(pg0, 0), a.n_pages - 1);
        pg1 = min(max(pg1, 0), a.n_pages - 1);
    }
    gmem_char* kp0 = st.k_head + (size_t)pg0 * page_bytes;
    gmem_char* kp1 = st.k_head + (size_t)pg1 * page_bytes;
    gmem_char* vp0 = st.v_head + (size_t)pg0 * page_bytes;
    gmem_char* vp1 = st.v_head + (size_t)pg1 * page_bytes;
    if constexpr (KV8) {
        const int kl = real ? li * ks + lg * 16 : 0;                  // K: key li, bytes 16 lg (+ 64 c)
        const int vl = real ? (lane >> 3) * ks + (lane & 7) * 16 : 0;  // V: key lane / 8 (+ 8 per r), chunk lane % 8
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            t.k[0][c] = tile_load<NT>((gmem_u32x4*)(kp0 + kl + 64 * c));
            t.k[1][c] = tile_load<NT>((gmem_u32x4*)(kp1 + kl + 64 * c));
        }
        t.v[0] = tile_load<NT>((gmem_u32x4*)(vp0 + vl));
        t.v[1] = tile_load<NT>((gmem_u32x4*)(vp0 + vl + 8 * ks));
        t.v[2] = tile_load<NT>((gmem_u32x4*)(vp1 + vl));
        t.v[3] = tile_load<NT>((gmem_u32x4*)(vp1 + vl + 8 * ks));
    } else {
        const int kl = real ? li * ks + lg * 16 : 0;  // K: key li, 16 bytes at d = 8 lg (+ 32 kk)
        const int vl = real ? lg * ks + li * 16 : 0;  // V: key lg (+ 4 r), 16-byte chunk li
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            if constexpr (KL) {  // lane copies 16-byte chunk li of keys 4 kk + lg: 1 KB of consecutive bytes per load
                t.k[0][kk] = __builtin_bit_cast(bf16x8, tile_load<NT>((gmem_s16x8*)(kp0 + vl + 4 * ks * kk)));
                t.k[1][kk] = __builtin_bit_cast(bf16x8, tile_load<NT>((gmem_s16x8*)(kp1 + vl + 4 * ks * kk)));
            } else {             // straight into the matrix operand's layout: 64 bytes out of each of 16 key rows per load
                t.k[0][kk] = __builtin_bit_cast(bf16x8, tile_load<NT>((gmem_s16x8*)(kp0 + kl + 64 * kk)));
                t.k[1][kk] = __builtin_bit_cast(bf16x8, tile_load<NT>((gmem_s16x8*)(kp1 + kl + 64 * kk)));
            }
        }
        // V: lane copies 16-byte chunk li of keys 4 r + lg, r = 0..7 (r >= 4: second page)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            t.v[r] = tile_load<NT>((gmem_s16x8*)(vp0 + vl + 4 * ks * r));
            t.v[4 + r] = tile_load<NT>((gmem_s16x8*)(vp1 + vl + 4 * ks * r));
        }
    }
}

// Process one segment: stream the wave's tiles, merge the waves, write the result or the partial.
// TEAMS = 1: the 4 waves split the keys and all work on the same (up to MT x 16) query rows.
// TEAMS = 2, for row groups wider than that: waves 0, 1 take the first per_team suffix positions and
// waves 2, 3 the rest, each pair splitting the keys between its two waves.  Both pairs read the same
// K/V bytes at about the same time, so HBM delivers them once (the second read is served by the L2
// of the workgroup's die) where two passes over the item would stream them twice.
template <int MT, bool TM, bool KV8, int RT, int TEAMS>
__device__ void attend_segment(const FastArgs& a, const Segment& sg, const KVStream& st, char* smem) {
    constexpr int kWPT = kWaves / TEAMS;  // waves that split the keys
    typedef Lds<RT, TEAMS == 2> L;
    // everything that is the same for the whole wave goes to scalar registers
    const int kvh = __builtin_amdgcn_readfirstlane(sg.kvh);
    const int c = __builtin_amdgcn_readfirstlane(sg.c);
    const int q0 = __builtin_amdgcn_readfirstlane(sg.q0);
    const int team = uniform(st.team), per_team = uniform(st.per_team);
    const int j0 = uniform(st.j0_t);        // the team's positions
    const int rows_g = uniform(st.rows_t);
    const bool final_out = sg.final_out;
    const int slot = sg.slot;
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wk = w % kWPT;
    const int lg = lane >> 4, li = lane & 15;
    const int G = a.G;
    const int M_g = G * rows_g;
    const int kv_total = uniform(st.kv_total), kb0 = uniform(st.kb0), nw = uniform(st.nw), step = uniform(st.step);
    char* kbuf = smem + w * L::kWaveRegion;  // the wave's K tile (where K goes through LDS), then its V tile
    char* vbuf = kbuf + kVTileBytes;

    const int vw_even = vtile_off(lg, li), vw_odd = vtile_off(4 + lg, li) - 4 * 256;  // LDS store offsets (+ 1024 r)
    // LDS transposed-read offsets: lane (lg, li) reads 8 bytes of key row 16 h + 4 lg + li/4 at
    // d = 16 db + 4 (li%4); after the transpose it holds keys 16 h + 4 lg + 0..3 at d = 16 db + li
    int vr_off[8];
    {
        const int r0 = 4 * lg + (li >> 2);
#pragma unroll
        for (int db = 0; db < 8; ++db) vr_off[db] = vtile_off(r0, 2 * db + ((li & 3) >> 1)) + (li & 1) * 8;
    }
    typedef typename TileOf<KV8>::type Tile;
    // Single-team segments over bf16 caches load K the way they load V -- whole key rows, 1 KB of consecutive
    // bytes per load -- and turn it into matrix operands through a wave-private LDS tile: non-temporal loads
    // that take 64 bytes out of each of 16 rows (K straight into the operand layout) fetch every line twice.
    // Measured, launch time with / without: 16-request shape 40.6 / 44.0 us, 128-request shape 253 / 263 us,
    // 512-request shape 1520 / 1533 us.  Two-team segments keep the direct K loads and the ordinary cache
    // policy: their second team's reads are meant to hit.
    constexpr bool KL = !KV8 && TEAMS == 1;
    auto issue = [&](Tile& t, int ti) { issue_tile<TM, KV8, false, TEAMS == 1, KL>(a, st, t, ti); };
    // with 8-bit caches the per-head key scale joins the softmax scale and the value scale the merge
    const float sl2 = KV8 ? a.scale_log2 * a.k_scale[kvh] : a.scale_log2;
    const float v_mul = KV8 ? a.v_scale[kvh] : 1.0f;
    // LDS store offsets of the 8-bit V path: key 8 r + lane / 8, the two bf16 chunks of its 16 bytes
    int v8_off[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) v8_off[r] = KV8 ? vtile_off(8 * r + (lane >> 3), 2 * (lane & 7)) : 0;
    // Two tiles in flight per wave.  (A third, where the registers would allow it, does not raise
    // the rate: a compute unit draws only about twice its even share of the HBM bandwidth however
    // much it keeps in flight.)
    constexpr int kDepth = 2;
    // ---- Q^T operands: lane holds query row (mt*16 + li), d = 32 kk + 8 lg .. +7.  They are the
    // same for the 4 waves and for every tile, so they live in LDS ([mt*4 + kk][lane] x 16 bytes,
    // read back lane-contiguous) instead of 16 registers per query tile.
    // Their loads go out BEFORE the K/V tiles': vector loads return in issue order, so query rows
    // sent for behind 32 KB of tiles would arrive only after the second tile, and every wave of the
    // workgroup would sit at the barrier below until then; sent for first they are staged while the
    // tiles travel, and the first tile is worked on as soon as it lands.
    char* qbuf = smem + L::kQ + (TEAMS == 2 ? team * kQTeamBytes : 0);
    int lim[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int m = mt * 16 + li;
        lim[mt] = m < M_g ? c + j0 + m / G : -1;
    }
    constexpr int kQPer = (MT * 4 + kWPT - 1) / kWPT;  // pieces of the team's operand buffer this wave brings in
    s16x8 q_piece[kQPer];
#pragma unroll
    for (int r = 0; r < kQPer; ++r) {
        const int pr = wk + r * kWPT;
        const int mt = pr >> 2, kk = pr & 3;
        const int m = mt * 16 + li;
        const bool ok = m < M_g && pr < MT * 4;
        const int j = j0 + m / G, gq = m % G;
        // the contraction index of matrix instruction kk, lane group lg covers d = 32 kk + 8 lg .. +7 with bf16
        // caches; with 8-bit ones a lane's 16-byte K chunk holds d = 64 c + 16 lg .. +15, split over kk = 2c, 2c+1
        const int d_off = KV8 ? 64 * (kk >> 1) + 16 * lg + 8 * (kk & 1) : 8 * lg + 32 * kk;
        const uint16_t* qp = a.q + ((size_t)(q0 + (ok ? j : j0)) * a.H_q + kvh * G + (ok ? gq : 0)) * kD + d_off;
        q_piece[r] = *reinterpret_cast<const s16x8*>(qp);
        if (!ok) q_piece[r] = s16x8{0, 0, 0, 0, 0, 0, 0, 0};
    }
    __builtin_amdgcn_sched_barrier(0);
    // (issued by every wave, also one without a tile of this segment: with no branch around them the
    // compiler's wait for the query rows counts exactly the loads behind them)
    Tile ta, tb;
    issue_tile<TM, KV8, true, TEAMS == 1, KL>(a, st, ta, 0);
    issue_tile<TM, KV8, true, TEAMS == 1, KL>(a, st, tb, 1);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int r = 0; r < kQPer; ++r) {
        const int pr = wk + r * kWPT;
        if (pr < MT * 4) *reinterpret_cast<s16x8*>(qbuf + (pr * 64 + lane) * 16) = q_piece[r];
    }
    __syncthreads();

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
    auto stage_and_scores = [&](Tile& t, int kb, f32x4 (&s)[MT][2]) {
        bf16x8 kop[2][4];  // K as matrix operands
        if constexpr (KV8) {
            // bytes -> bf16 in registers (exact), then everything is as with a bf16 cache
            if (kb + kTile > kv_total) {  // slots past the request's last token may hold anything: zero them
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    if (kb + 8 * r + (lane >> 3) >= kv_total) t.v[r] = u32x4{0u, 0u, 0u, 0u};
            }
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                u32x4 lo8, hi8;
                e4m3x16_to_bf16(t.v[r], lo8, hi8);
                *reinterpret_cast<u32x4*>(vbuf + v8_off[r]) = lo8;
                *reinterpret_cast<u32x4*>(vbuf + v8_off[r] + 16) = hi8;
            }
#pragma unroll
            for (int pg = 0; pg < 2; ++pg)
#pragma unroll
                for (int c = 0; c < 2; ++c) {
                    u32x4 lo8, hi8;
                    e4m3x16_to_bf16(t.k[pg][c], lo8, hi8);
                    kop[pg][2 * c] = __builtin_bit_cast(bf16x8, lo8);
                    kop[pg][2 * c + 1] = __builtin_bit_cast(bf16x8, hi8);
                }
        } else {
            if (kb + kTile > kv_total) {  // slots past the request's last token may hold anything: zero them
#pragma unroll
                for (int r = 0; r < 8; ++r)
                    if (kb + 4 * r + lg >= kv_total) t.v[r] = s16x8{0, 0, 0, 0, 0, 0, 0, 0};
            }
#pragma unroll
            for (int r = 0; r < 8; ++r)
                *reinterpret_cast<s16x8*>(vbuf + ((r & 1) ? vw_odd : vw_even) + 1024 * r) = t.v[r];
            if constexpr (KL) {
                // K tile in LDS: rows of 256 bytes, chunk c of row i at slot c ^ i (16 lanes that write one row's chunks,
                // or read one chunk of 16 rows, cover all the banks); read back as matrix operands: lane (li, lg) takes
                // chunk 4 kk + lg of row li
#pragma unroll
                for (int pg = 0; pg < 2; ++pg)
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        *reinterpret_cast<bf16x8*>(kbuf + 4096 * pg + (4 * r + lg) * 256 + ((li ^ (4 * r + lg)) << 4)) = t.k[pg][r];
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
                for (int pg = 0; pg < 2; ++pg)
#pragma unroll
                    for (int kk = 0; kk < 4; ++kk)
                        kop[pg][kk] = *reinterpret_cast<const bf16x8*>(kbuf + 4096 * pg + li * 256 + (((4 * kk + lg) ^ li) << 4));
            } else {
#pragma unroll
                for (int pg = 0; pg < 2; ++pg)
#pragma unroll
                    for (int kk = 0; kk < 4; ++kk) kop[pg][kk] = t.k[pg][kk];
            }
        }
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
                s[mt][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kop[0][kk], qop[mt][kk], s[mt][0], 0, 0, 0);
                s[mt][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kop[1][kk], qop[mt][kk], s[mt][1], 0, 0, 0);
            }
        }
        if constexpr (!KL) {
            __builtin_amdgcn_sched_group_barrier(0x200, 8, 0);       // V stores
            __builtin_amdgcn_sched_group_barrier(0x100, 4 * MT, 0);  // Q^T operand reads
            __builtin_amdgcn_sched_group_barrier(0x008, 8 * MT, 0);  // score MFMAs
        }
    };

    // raw scores of all query tiles with the keys a row may not see set to -inf
    // (may_mask = false: the caller knows that every row sees every key of the tile)
    auto masked_scores = [&](int kb, const f32x4 (&s)[MT][2], float (&x)[MT][8], bool may_mask = true) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                for (int e = 0; e < 4; ++e) x[mt][kt * 4 + e] = s[mt][kt][e];
        if (may_mask && kb + kTile > c + j0 + 1) {  // only the item's last keys are causal-masked or past the end
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
        if constexpr (!KL) {  // (the K tile's round trip through LDS has ordered the V stores too)
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        }
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
            const float p0 = fast_exp2(fmaf(x[e], sl2, neg_m)), p1 = fast_exp2(fmaf(x[e + 1], sl2, neg_m));
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
    auto fast_softmax_pv = [&](int kb, const f32x4 (&s)[MT][2], bool may_mask) {
        bf16x8 vop[8];
        load_vops(vop);
        float x[MT][8], lane_max[MT];
        masked_scores(kb, s, x, may_mask);
        bool any = false;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            lane_max[mt] = sl2 * max8(x[mt]);
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
        // one tile: wait for it, stage V, scores; softmax and P V; then refill its registers with the
        // tile kDepth further on (past the end: a harmless repeat of the last tile).  The refill goes out
        // after the tile's arithmetic, not before it: HBM is saturated either way, and the fewer bytes the
        // chip keeps queued the sooner a segment's first tiles, its partials and its arrival count come back
        // (measured: 0.2 to 0.7 % per launch on every workload shape).
        auto fast_tile = [&](Tile& tl, int t, auto plain) {
            const bool real = t < nw;
            if (real) stage_and_scores(tl, kb0 + t * step, s);
            __builtin_amdgcn_sched_barrier(0);
            if (real) fast_softmax_pv(kb0 + t * step, s, !decltype(plain)::value);
            __builtin_amdgcn_sched_barrier(0);
            issue(tl, t + kDepth);
            __builtin_amdgcn_sched_barrier(0);
        };
        // The wave's first n_plain tiles lie wholly below the first row's causal limit (every row sees every
        // key): pairs of them run a loop with no masking code in it -- as a select per score inside the one loop
        // it cost a third of the loop's vector instructions, most of them copies between the two register
        // files -- and the rest, the item's last few tiles, the general loop.
        const int below = c + j0 + 1 - kTile - kb0;  // tile t is plain iff t * step <= below
        const int n_plain = below < 0 ? 0 : min(below / step + 1, nw);
        int t = 0;
        for (; t + 1 < n_plain; t += kDepth) {
            fast_tile(ta, t, std::true_type{});
            fast_tile(tb, t + 1, std::true_type{});
        }
        for (; t < nw; t += kDepth) {
            fast_tile(ta, t, std::false_type{});
            fast_tile(tb, t + 1, std::false_type{});
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
        auto issue_one = [&](Tile& t, int ti) {
            if (ti < nw) issue(t, ti);
        };
        auto needs_raise = [&](int kb, const f32x4 (&s)[MT][2]) {
            bool any = false;
            float x[MT][8];
            masked_scores(kb, s, x);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) any |= sl2 * max8(x[mt]) > m_run[mt] + kSlack;
            return __builtin_amdgcn_ballot_w64(any) != 0;
        };
        auto raise_refs = [&](int kb, const f32x4 (&s)[MT][2]) {
            float x[MT][8];
            masked_scores(kb, s, x);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                const float lane_max = sl2 * max8(x[mt]);
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
            raise_refs(kb0 + t * step, s);
            for (;;) {
                exact_softmax_pv(kb0 + t * step, s);
                if (++t >= nw) {
                    more = false;
                    break;
                }
                stage_and_scores(ta, kb0 + t * step, s);
                issue_one(ta, t + 1);
                if (needs_raise(kb0 + t * step, s)) break;
            }
        }
    }

    // ---- row sums live spread over the 4 lane groups
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        l_run[mt] += __shfl_xor(l_run[mt], 16, 64);
        l_run[mt] += __shfl_xor(l_run[mt], 32, 64);
    }

    // ---- merge the waves of each team (each saw a disjoint set of keys).  A wave puts its exponent references,
    // its sums and its accumulators, as they are, into its own LDS region as soon as its own loop is over (the
    // region held its K/V tiles, which are dead by then; nobody else touches it), so that after the barrier that
    // waits for the slowest wave only the sums are left to do; the weights exp2(reference - row maximum) are
    // applied there.
    float* red_m = reinterpret_cast<float*>(smem + L::kMl);  // [kWaves][16 * kMaxMT]
    float* red_l = red_m + kWaves * 16 * kMaxMT;
    constexpr int kTileFloats = 16 * kRedStride;  // one query tile of one wave
    float* red_own = reinterpret_cast<float*>(smem + w * L::kWaveRegion);
    const __amdgpu_buffer_rsrc_t buf_o = partial_buffer(a.part_o), buf_ml = partial_buffer(a.part_ml);
    if (lg == 0) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            red_m[w * 16 * kMaxMT + mt * 16 + li] = m_run[mt];
            red_l[w * 16 * kMaxMT + mt * 16 + li] = l_run[mt];
        }
    }
    auto dump_batch = [&](int mt0) {
#pragma unroll
        for (int r = 0; r < RT; ++r) {
            const int mt = mt0 + r;
            if (mt >= MT) break;
#pragma unroll
            for (int db = 0; db < 8; ++db)
                *reinterpret_cast<f32x4*>(red_own + r * kTileFloats + li * kRedStride + db * 16 + 4 * lg) = acc[mt][db];
        }
    };
    dump_batch(0);
    __syncthreads();
#pragma unroll
    for (int mt0 = 0; mt0 < MT; mt0 += RT) {
        if (mt0 > 0) {
            dump_batch(mt0);
            __syncthreads();
        }
        // 256 threads sum 16 rows x 128 d over the waves of a team: thread -> row tid/16, 8 consecutive d
#pragma unroll
        for (int tt = 0; tt < TEAMS; ++tt) {
            // the rows of team tt (every thread sums for both teams, whichever its own wave belongs to)
            const int j0_s = TEAMS == 1 ? j0 : uniform(sg.j0) + tt * per_team;
            const int rows_s = TEAMS == 1 ? rows_g : tt == 0 ? min(uniform(sg.rows_g), per_team) : uniform(sg.rows_g) - per_team;
            const int M_s = G * rows_s, ws0 = tt * kWPT;
#pragma unroll
            for (int r = 0; r < RT; ++r) {
                const int mt = mt0 + r;
                if (mt >= MT) break;
                const int row = threadIdx.x >> 4, d0 = (threadIdx.x & 15) * 8;
                const int m = mt * 16 + row;
                // every LDS read of the tile is sent for before the first sum: one wait instead of one per pair
                // of reads (a wave runs alone on its SIMD, nothing else hides the LDS latency)
                f32x4 part0[kWPT], part1[kWPT];
                float wm[kWPT], wl[kWPT];
#pragma unroll
                for (int ww = 0; ww < kWPT; ++ww) {
                    const float* red_w = reinterpret_cast<const float*>(smem + (ws0 + ww) * L::kWaveRegion) + r * kTileFloats;
                    part0[ww] = *reinterpret_cast<const f32x4*>(red_w + row * kRedStride + d0);
                    part1[ww] = *reinterpret_cast<const f32x4*>(red_w + row * kRedStride + d0 + 4);
                    wm[ww] = red_m[(ws0 + ww) * 16 * kMaxMT + m];
                    wl[ww] = red_l[(ws0 + ww) * 16 * kMaxMT + m];
                }
                __builtin_amdgcn_sched_barrier(0);
                float ms = -INFINITY;
#pragma unroll
                for (int ww = 0; ww < kWPT; ++ww) ms = fmaxf(ms, wm[ww]);
                const float mu = ms == -INFINITY ? 0.0f : ms;
                f32x4 s0 = f32x4{0.f, 0.f, 0.f, 0.f}, s1 = s0;
                float ls = 0.0f;
#pragma unroll
                for (int ww = 0; ww < kWPT; ++ww) {
                    const float e = fast_exp2(wm[ww] - mu);  // weight of the wave's piece (0 for a wave that saw no key of the row)
                    ls += wl[ww] * e;
                    s0 += part0[ww] * (e * v_mul);
                    s1 += part1[ww] * (e * v_mul);
                }
                if (m < M_s) {
                    if (final_out) {
                        const int j = j0_s + m / G, h = kvh * G + m % G;
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
                        // pieces are read by another workgroup of this launch, possibly on another die:
                        // device-coherent stores (written through to memory) instead of a cache flush before the count.
                        // A slot holds the row group's rows in order: the second team's behind the first's.
                        const size_t prow = (size_t)slot * a.m_cap + tt * G * per_team + m;
                        coherent_store4(buf_o, prow * kD + d0, s0);
                        coherent_store4(buf_o, prow * kD + d0 + 4, s1);
                        if (d0 == 0) coherent_store4(buf_ml, prow * 4, f32x4{ms, ls, __builtin_bit_cast(float, (uint32_t)a.call_id), 0.0f});
                    }
                }
            }
        }
        __syncthreads();
    }
}

// Stream, attend and merge one segment with the kernel variant its row group needs.
template <int MTMAX, bool TM, bool KV8, int RT, bool WIDE>
__device__ __forceinline__ void attend_dispatch(const FastArgs& a, const Segment& sg, char* smem, bool rec_pages, int pgv) {
    const int per_team = rows_per_team(a, MTMAX);
    if constexpr (WIDE) {
        static_assert(MTMAX == kWideMT, "two-team segments are built for three query tiles per team");
        if (sg.rows_g > per_team) {
            KVStream st = make_stream<TM, KV8>(a, sg, per_team, 2);
            st.rec_pages = rec_pages;
            st.pgv = pgv;
            attend_segment<MTMAX, TM, KV8, RT, 2>(a, sg, st, smem);
            return;
        }
    }
    KVStream st = make_stream<TM, KV8>(a, sg, per_team, 1);
    st.rec_pages = rec_pages;
    st.pgv = pgv;
    const int mt = (a.G * sg.rows_g + 15) >> 4;
#define FSR_SEG(MT) attend_segment<MT, TM, KV8, RT, 1>(a, sg, st, smem)
    if constexpr (MTMAX == 1) {
        FSR_SEG(1);
    } else if constexpr (MTMAX == 2) {
        if (mt == 1) FSR_SEG(1); else FSR_SEG(2);
    } else if constexpr (MTMAX == 3) {
        if (mt == 1) FSR_SEG(1); else if (mt == 2) FSR_SEG(2); else FSR_SEG(3);
    } else {
        static_assert(MTMAX == 4, "kernels are built for 1 to 4 query tiles");
        if (mt <= 2) FSR_SEG(2); else if (mt == 3) FSR_SEG(3); else FSR_SEG(4);
    }
#undef FSR_SEG
}

// Combine the pieces of an item that share boundaries cut: slot 1 of workgroup b_first (which holds
// the item's first tile) and slot 0 of b_first+1 .. b_last.  Called by one whole workgroup.  A thread
// owns up to kE (row, 4 d) elements and has the loads of all of them, for two pieces at a time, in
// flight together: the pieces come from the point of coherence, a long way off.  q0 = output row of
// the item's first suffix position.
template <int MTMAX>
__device__ void combine_cut_item(const FastArgs& a, int b_first, int b_last, int g, int q0, int M) {
    constexpr int kE = (16 * MTMAX * (kD / 4) + kThreads - 1) / kThreads;
    constexpr int kBatch = 2;
    const int n_elem = M * (kD / 4);
    // a row group of two teams holds up to twice 16 * MTMAX rows: a second round over the pieces
    for (int e_base = 0; e_base < n_elem; e_base += kE * kThreads) {
        float m_star[kE], l[kE];
        f32x4 o[kE];
#pragma unroll
        for (int e = 0; e < kE; ++e) {
            m_star[e] = -INFINITY;
            l[e] = 0.0f;
            o[e] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
        for (int bb0 = b_first; bb0 <= b_last; bb0 += kBatch) {
            float pm[kE][kBatch], pl[kE][kBatch];
            f32x4 po[kE][kBatch];
#pragma unroll
            for (int e = 0; e < kE; ++e) {
                const int idx = min(e_base + (int)threadIdx.x + e * kThreads, n_elem - 1);  // past the end: a valid element, unused
                const int m = idx / (kD / 4), d0 = (idx % (kD / 4)) * 4;
#pragma unroll
                for (int k = 0; k < kBatch; ++k) {
                    const int bb = min(bb0 + k, b_last);  // past the end: the last piece again, weighted 0 below
                    const size_t row = (size_t)(bb * 2 + (bb == b_first ? 1 : 0)) * a.m_cap + m;
                    // Ordinary loads are enough on this side (and 0.5 us quicker than device-coherent ones): a piece
                    // was stored through to memory and acknowledged before it was counted; a slot is written once and
                    // read once per launch, so neither this compute unit's L1 nor this die's L2 can hold an older copy
                    // of it from this launch, and copies from earlier launches are dropped when a kernel starts (the same
                    // rule that lets any kernel read what an earlier kernel wrote on another die).
                    const f32x4 ml4 = *reinterpret_cast<const f32x4*>(a.part_ml + row * 4);
                    // a slot that this call did not write (a workspace shared by overlapping calls) poisons the row
                    // instead of being summed silently
                    const float ref = ml4[0], sum = ml4[1], tag = ml4[2];
                    pm[e][k] = __builtin_bit_cast(uint32_t, tag) == (uint32_t)a.call_id ? ref : __builtin_nanf("");
                    pl[e][k] = sum;
                    po[e][k] = *reinterpret_cast<const f32x4*>(a.part_o + row * kD + d0);
                }
            }
#pragma unroll
            for (int e = 0; e < kE; ++e) {
                float m_new = m_star[e];
#pragma unroll
                for (int k = 0; k < kBatch; ++k)
                    if (bb0 + k <= b_last) m_new = fmaxf(m_new, pm[e][k]);
                const float mu = m_new == -INFINITY ? 0.0f : m_new;
                const float keep = fast_exp2(m_star[e] - mu);  // 0 while nothing has been accumulated
                l[e] *= keep;
                o[e] *= keep;
#pragma unroll
                for (int k = 0; k < kBatch; ++k) {
                    const float wgt = bb0 + k <= b_last ? fast_exp2(pm[e][k] - mu) : 0.0f;
                    l[e] += pl[e][k] * wgt;
                    o[e] += po[e][k] * wgt;
                }
                m_star[e] = m_new;
            }
        }
#pragma unroll
        for (int e = 0; e < kE; ++e) {
            const int idx = e_base + threadIdx.x + e * kThreads;
            if (idx >= n_elem) break;
            const int m = idx / (kD / 4), d0 = (idx % (kD / 4)) * 4;
            const f32x4 r = o[e] * (1.0f / l[e]);
            const int j = m / a.G, h = g * a.G + m % a.G;
            const size_t o_idx = ((size_t)(q0 + j) * a.H_q + h) * kD + d0;
            if (a.out_bf16) {
                ushort4 pk;
                pk.x = f32_to_bf16_rne(r[0]);
                pk.y = f32_to_bf16_rne(r[1]);
                pk.z = f32_to_bf16_rne(r[2]);
                pk.w = f32_to_bf16_rne(r[3]);
                *reinterpret_cast<ushort4*>(reinterpret_cast<uint16_t*>(a.out) + o_idx) = pk;
            } else {
                *reinterpret_cast<f32x4*>(reinterpret_cast<float*>(a.out) + o_idx) = r;
            }
            if (a.lse && d0 == 0) a.lse[(size_t)(q0 + j) * a.H_q + h] = (m_star[e] + __log2f(l[e])) * kLn2;
        }
    }
}

// After a segment that is a piece of a cut item: count the piece; the workgroup whose piece arrives
// last combines them all.  Called by the whole workgroup.
template <int MTMAX>
__device__ __forceinline__ void finish_piece(const FastArgs& a, const Segment& sg, int* s_last) {
    // the piece's stores are device-coherent; once every wave has seen them acknowledged the piece
    // may be counted
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (threadIdx.x == 0) *s_last = count_arrival(a.arrivals + sg.b_first + 1, a.call_id) == sg.b_last - sg.b_first + 1;
    __syncthreads();
    if (*s_last) {
        combine_cut_item<MTMAX>(a, sg.b_first, sg.b_last, sg.kvh, sg.q0 + sg.j0, a.G * sg.rows_g);
        if (threadIdx.x == 0) __atomic_store_n(a.arrivals + sg.b_first + 1, a.call_id << 16, __ATOMIC_RELAXED);
    }
    __syncthreads();
}

// Persistent grid: nb workgroups of 256 threads; the cost line [0, T) is cut into nb' = min(nb,
// T / dearest tile) shares whose lengths differ by at most one unit, every workgroup takes one share.  A
// share owns the tiles that END inside it (phantom tiles are owned and skipped).  An item that lies
// inside one share is finished by that workgroup; an item cut by share boundaries leaves one
// partial per piece, and the workgroup whose piece arrives last combines them (no workgroup ever
// waits for another).
//
// attn_stream_kernel builds the schedule itself, from the lengths, at the start of every launch.
template <int MTMAX, bool TM, bool KV8, bool WIDE>
__global__ __launch_bounds__(kThreads) void attn_stream_kernel(FastArgs a) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    __shared__ int s_last;
    char* tables = smem + stream_fixed_smem(WIDE);
    long long* pref = reinterpret_cast<long long*>(tables);
    const int cmax = build_cost_prefix(a, MTMAX, pref, reinterpret_cast<long long*>(tables + scan_off(a.B)),
                                       reinterpret_cast<int*>(tables + cu_off(a.B)), reinterpret_cast<int*>(tables + ctx_off(a.B)));
    ShareWalker<true> wk;
    wk.pref = pref;
    wk.lds_cu = reinterpret_cast<const int*>(tables + cu_off(a.B));
    wk.lds_ctx = reinterpret_cast<const int*>(tables + ctx_off(a.B));
    // every share is at least as wide as the dearest tile: a workgroup whose share lies inside an
    // item then owns at least one of its tiles
    const long long total = pref[a.B] * a.H_kv;
    const int nbx = (int)min((long long)a.nb, div_u(total, cmax));
    wk.b = share_of_block(blockIdx.x, a.nb);
    if (wk.b >= nbx) return;
    wk.set_shares(total, nbx);
    wk.mt_max = MTMAX;
    wk.x = wk.share_start(wk.b);
    wk.x1 = wk.share_start(wk.b + 1);

    Segment cur;
    while (wk.next(a, cur)) {
        attend_dispatch<MTMAX, TM, KV8, kStreamRT, WIDE>(a, cur, smem, false, 0);
        if (cur.cut) finish_piece<MTMAX>(a, cur, &s_last);
    }
}

// ---------------------------------------------------------------------------------------
// Planned schedule.  Lengths, row offsets and block tables are the same for every layer of a
// verification step, so the schedule can be built once per step (attn_plan_kernel) and the
// per-layer launches (attn_planned_kernel) then start their first K/V loads one scalar-load round
// trip after they begin: a workgroup reads the record of its first segment, which also carries the
// page ids of the first two tiles of each of its waves.
//
// Plan buffer (int32 words): header record, then one record per share (its first segment), then the
// further segments of all shares, share after share.  A record is kRecInts words:
//   0 request  1 KV head  2 context  3 first row  4 rows of the request  5 first suffix position of
//   the row group  6 positions in the group  7,8 tile range  9 flags (1 = whole item, 2 = cut)
//   10,11 first / last share of the cut item  12 partial slot  13 segments of this share (first
//   record only)  14 index of the share's second segment among the further ones (first record only)
//   16..31 page ids of the item's tiles tile_a .. tile_a + 7 (two pages each, clamped to the pool and
//   to the request's last page)
// Header: 0 magic, 1 key of the shapes the plan was built for, 2 shares in use.
// ---------------------------------------------------------------------------------------
constexpr int kRecInts = 32;
constexpr int kMaxShares = 1024;  // the workspace and the plan are laid out for up to this many workgroups
constexpr int32_t kPlanMagic = 0x46535250;

__device__ __forceinline__ void write_record(int32_t* rec, const FastArgs& a, const Segment& sg, int n_seg, int more_at) {
    int32_t w[kRecInts];
    w[0] = sg.i; w[1] = sg.kvh; w[2] = sg.c; w[3] = sg.q0; w[4] = sg.q_len; w[5] = sg.j0; w[6] = sg.rows_g;
    w[7] = sg.tile_a; w[8] = sg.tile_e; w[9] = (sg.final_out ? 1 : 0) | (sg.cut ? 2 : 0);
    w[10] = sg.b_first; w[11] = sg.b_last; w[12] = sg.slot; w[13] = n_seg; w[14] = more_at; w[15] = 0;
    const int kv_total = min(sg.c + sg.q_len, a.max_pages * kP);
    const int last_page = max((kv_total + kP - 1) / kP - 1, 0);
    const int32_t* bt = a.bt + (size_t)sg.i * a.max_pages;
#pragma unroll
    for (int k = 0; k < 16; ++k) w[16 + k] = min(max(bt[min(2 * sg.tile_a + k, last_page)], 0), a.n_pages - 1);
#pragma unroll
    for (int k = 0; k < kRecInts; k += 4) *reinterpret_cast<int4*>(rec + k) = make_int4(w[k], w[k + 1], w[k + 2], w[k + 3]);
}

// One workgroup; thread t walks shares t, t + 256, ... twice (count, then write).
__global__ __launch_bounds__(kThreads) void attn_plan_kernel(FastArgs a, int mt_max, int32_t* plan, int more_cap) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    long long* pref = reinterpret_cast<long long*>(smem);
    long long* scratch = reinterpret_cast<long long*>(smem + scan_off(a.B));
    int* cnt = reinterpret_cast<int*>(smem + tables_bytes(a.B));  // [kMaxShares] segments of a share, then where its further ones start
    const int cmax = build_cost_prefix(a, mt_max, pref, scratch, reinterpret_cast<int*>(smem + cu_off(a.B)),
                                       reinterpret_cast<int*>(smem + ctx_off(a.B)));
    ShareWalker<false> wk;
    wk.pref = pref;
    wk.lds_cu = reinterpret_cast<const int*>(smem + cu_off(a.B));
    wk.lds_ctx = reinterpret_cast<const int*>(smem + ctx_off(a.B));
    wk.mt_max = mt_max;
    const long long total = pref[a.B] * a.H_kv;
    const int nbx = (int)min((long long)a.nb, div_u(total, cmax));
    if (nbx > 0) wk.set_shares(total, nbx);
    for (int s = threadIdx.x; s < kMaxShares; s += kThreads) {
        int n = 0;
        if (s < nbx) {
            wk.b = s; wk.x = wk.share_start(s); wk.x1 = wk.share_start(s + 1);
            Segment sg;
            while (wk.next(a, sg)) ++n;
        }
        cnt[s] = n;
    }
    __syncthreads();
    // exclusive scan of max(cnt - 1, 0): thread t owns shares 4 t .. 4 t + 3
    {
        const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
        int mine[4], sum = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            mine[j] = sum;
            sum += max(cnt[4 * threadIdx.x + j] - 1, 0);
        }
        const int inc = wave_inclusive_scan(sum);
        __syncthreads();  // every count has been read; the table is reused for the offsets
        if (lane == 63) scratch[w] = inc;
        __syncthreads();
        int before = 0;
#pragma unroll
        for (int k = 0; k < kWaves; ++k)
            if (k < w) before += (int)scratch[k];
#pragma unroll
        for (int j = 0; j < 4; ++j) cnt[4 * threadIdx.x + j] = before + inc - sum + mine[j];
        __syncthreads();
    }
    int32_t* first = plan + kRecInts;
    int32_t* more = first + (size_t)kMaxShares * kRecInts;
    for (int s = threadIdx.x; s < a.nb; s += kThreads) {
        const int more_at = cnt[s];
        int n = 0;
        Segment sg, head;
        if (s < nbx) {
            wk.b = s; wk.x = wk.share_start(s); wk.x1 = wk.share_start(s + 1);
            while (wk.next(a, sg)) {
                if (n == 0) head = sg;
                else if (more_at + n - 1 < more_cap) write_record(more + (size_t)(more_at + n - 1) * kRecInts, a, sg, 0, 0);
                else break;  // cannot happen with the capacity the host computes; stay inside the buffer anyway
                ++n;
            }
        }
        if (n > 0) {
            write_record(first + (size_t)s * kRecInts, a, head, n, more_at);
        } else {
            first[(size_t)s * kRecInts + 13] = 0;
        }
    }
    if (threadIdx.x == 0) {
        plan[2] = nbx;
        plan[1] = (int32_t)a.plan_key;
        plan[0] = kPlanMagic;
    }
}

template <int MTMAX, bool TM, bool KV8, bool WIDE>
__global__ __launch_bounds__(kThreads) void attn_planned_kernel(FastArgs a) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    __shared__ int s_last;
    const const_i32* plan = (const const_i32*)a.plan;
    const int share = share_of_block(blockIdx.x, a.nb);
    const const_i32* rec = plan + (size_t)(1 + share) * kRecInts;
    // Header and first record are sent for together, before anything is known about either (the record's
    // address lies inside the plan buffer whatever the buffer holds): the fields through the scalar cache,
    // the sixteen page ids as one vector load, lane l holding entry l % 16.  One round trip after the
    // kernel starts the workgroup can send for its query rows and first tiles.
    const int lane16 = threadIdx.x & 15;
    int magic = plan[0], key = plan[1];
    int f[16];
#pragma unroll
    for (int k = 0; k < 16; ++k) f[k] = rec[k];
    int pgv = a.plan[(size_t)(1 + share) * kRecInts + 16 + lane16];
    // a buffer that holds no plan, or one built for other shapes, is left alone (the host checks the
    // shapes before the launch; this guards the memory accesses below)
    if (magic != kPlanMagic || key != (int32_t)a.plan_key) return;
    const int n_seg = f[13];
    const size_t more_rec = (size_t)1 + kMaxShares + f[14];
    for (int k = 0; k < n_seg; ++k) {
        if (k > 0) {
            rec = plan + (more_rec + k - 1) * kRecInts;
#pragma unroll
            for (int j = 0; j < 13; ++j) f[j] = rec[j];
            pgv = a.plan[(more_rec + k - 1) * kRecInts + 16 + lane16];
        }
        Segment cur;
        cur.i = f[0]; cur.kvh = f[1]; cur.c = f[2]; cur.q0 = f[3]; cur.q_len = f[4]; cur.j0 = f[5];
        cur.rows_g = f[6]; cur.tile_a = f[7]; cur.tile_e = f[8];
        const int flags = f[9];
        cur.final_out = (flags & 1) != 0; cur.cut = (flags & 2) != 0;
        cur.b_first = f[10]; cur.b_last = f[11]; cur.slot = f[12];
        attend_dispatch<MTMAX, TM, KV8, MTMAX, WIDE>(a, cur, smem, true, pgv);
        if (cur.cut) finish_piece<MTMAX>(a, cur, &s_last);
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
    int token_major;  // 1: caches are [page][P][H_kv][D], 0: [page][H_kv][P][D]
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
        const size_t base = a.token_major ? (((size_t)pg * a.P + t % a.P) * a.H_kv + g) * D
                                          : (((size_t)pg * a.H_kv + g) * a.P + t % a.P) * D;
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

// How a call is run.
struct Setup {
    bool fast;   // the stream kernel (bf16, D = 128, P = 16, G <= 16, B <= kMaxB); else one wave per (row, head)
    int mt_max;  // 16-row query tiles a team of waves takes (template argument of the kernel)
    bool wide;   // row groups of two teams (requests with more than kMaxMT query tiles of rows per KV head)
    int m_cap;   // rows a partial slot holds
    int nb;      // workgroups of the persistent grid
    int shares_cap;  // shares the workspace is laid out for
    size_t bytes_o, bytes_ml, bytes_cnt;
    size_t ws_bytes() const { return bytes_o + bytes_ml + bytes_cnt; }
};

int validate(const fsr_attn_params* p, const char* who) {
    if (!p) return fail(FSR_EINVAL, "%s: params is null", who);
    if (p->max_q_len < 0) return fail(FSR_EINVAL, "%s: max_q_len=%d", who, p->max_q_len);
    if (p->B < 0 || p->N_cap < 0 || p->H_q <= 0 || p->H_kv <= 0 || p->max_pages <= 0 || p->n_pages <= 0 || p->P <= 0 || p->max_workgroups < 0 ||
        (p->kv_layout != FSR_KV_HEAD_MAJOR && p->kv_layout != FSR_KV_TOKEN_MAJOR))
        return fail(FSR_EINVAL, "%s: B=%d N_cap=%d H_q=%d H_kv=%d max_pages=%d n_pages=%d P=%d max_workgroups=%d kv_layout=%d", who, p->B, p->N_cap,
                    p->H_q, p->H_kv, p->max_pages, p->n_pages, p->P, p->max_workgroups, p->kv_layout);
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

// shares_cap: what the partial slots and arrival words are laid out for (the workspace of the ordinary
// entry points is sized for kMaxShares so that its size does not depend on the device).
Setup make_setup(const fsr_attn_params& p, int shares_cap = kMaxShares) {
    Setup su{};
    const int G = p.H_q / p.H_kv;
    su.fast = p.dtype == FSR_BF16 && p.D == kD && p.P == kP && G <= 16 && p.B <= kMaxB;
    if (!su.fast) return su;
    // rows of one request that share a KV head: G * max_q_len (unknown bound -> the widest kernel)
    // When they fit four query tiles they are one row group; beyond that (or with no bound given) a
    // request is cut into row groups of up to three tiles, the widest kernel that keeps its
    // accumulators and both K/V tiles in registers without spilling.
    const long long m_rows = p.max_q_len > 0 ? (long long)G * p.max_q_len : 1 << 20;
    const long long mt = (m_rows + 15) / 16;
    su.wide = mt > kMaxMT;
    su.mt_max = su.wide ? kWideMT : (int)mt;
    su.m_cap = 16 * su.mt_max * (su.wide ? 2 : 1);
    su.shares_cap = shares_cap;
    su.nb = std::min(persistent_blocks(), shares_cap);
    if (p.max_workgroups > 0) su.nb = std::min(su.nb, p.max_workgroups);
    su.bytes_o = align_up((size_t)shares_cap * 2 * su.m_cap * kD * sizeof(float), 256);
    su.bytes_ml = align_up((size_t)shares_cap * 2 * su.m_cap * 4 * sizeof(float), 256);
    su.bytes_cnt = align_up((size_t)(shares_cap + 1) * sizeof(unsigned long long), 256);
    return su;
}

int cost_base_for(const fsr_attn_params& p, const Setup& su) {
    return (int)std::min<long long>(kCostBaseMax, std::max<long long>(kCostBase, 2LL * p.B * p.H_kv / su.nb));
}

// What a plan depends on besides the device arrays it was built from.
uint32_t plan_key_of(const fsr_attn_params& p, const Setup& su) {
    uint32_t h = 2166136261u;
    const int v[] = {p.B, p.N_cap, p.H_q, p.H_kv, p.max_pages, p.n_pages, su.mt_max, su.wide ? 1 : 0, su.nb, cost_base_for(p, su), kSegTiles};
    for (int x : v) {
        h = (h ^ (uint32_t)x) * 16777619u;
        h ^= h >> 15;
    }
    return h | 1u;
}

// Segments beyond a share's first that any batch of these shapes can have: every item contributes one
// segment per share it touches, i.e. at most (items + shares) segments in all.
size_t plan_more_cap(const fsr_attn_params& p, const Setup& su) {
    const int G = p.H_q / p.H_kv;
    const long long per_group = std::max(16 * su.mt_max / G, 1) * (su.wide ? 2 : 1);
    const long long items = (long long)p.H_kv * ((long long)p.B + p.N_cap / per_group + 1);
    return (size_t)(items + kMaxShares);
}
size_t plan_bytes_of(const fsr_attn_params& p, const Setup& su) {
    return (size_t)(1 + kMaxShares + plan_more_cap(p, su)) * kRecInts * sizeof(int32_t);
}

// Plans this process has built: device address -> key.  A host-side record, so that a call handed a
// buffer that holds no plan, or a plan for other shapes, is refused before anything is launched.
std::mutex g_plans_mutex;
std::map<const void*, uint32_t> g_plans;

}  // namespace
}  // namespace fsr

using namespace fsr;

extern "C" int fsr_attn_workspace_bytes(const fsr_attn_params* p, size_t* out_bytes) {
    int rc = validate(p, "fsr_attn_workspace_bytes");
    if (rc != FSR_OK) return rc;
    if (!out_bytes) return fail(FSR_EINVAL, "fsr_attn_workspace_bytes: out_bytes is null");
    const Setup su = make_setup(*p);
    *out_bytes = su.fast ? su.ws_bytes() : 0;
    return FSR_OK;
}

extern "C" int fsr_attn_path(const fsr_attn_params* p) {
    int rc = validate(p, "fsr_attn_path");
    if (rc != FSR_OK) return rc;
    return make_setup(*p).fast ? FSR_PATH_STREAM : FSR_PATH_GENERIC;
}

extern "C" int fsr_attn_plan_bytes(const fsr_attn_params* p, size_t* out_bytes) {
    int rc = validate(p, "fsr_attn_plan_bytes");
    if (rc != FSR_OK) return rc;
    if (!out_bytes) return fail(FSR_EINVAL, "fsr_attn_plan_bytes: out_bytes is null");
    const Setup su = make_setup(*p);
    *out_bytes = su.fast ? plan_bytes_of(*p, su) : 0;
    return FSR_OK;
}

namespace {
void fill_common(FastArgs& a, const fsr_attn_params* p, const Setup& su, const int32_t* block_tables, const int32_t* ctx_lens,
                 const int32_t* cu_q) {
    a.bt = block_tables; a.ctx = ctx_lens; a.cu_q = cu_q;
    a.B = p->B; a.H_q = p->H_q; a.H_kv = p->H_kv; a.G = p->H_q / p->H_kv;
    a.max_pages = p->max_pages; a.n_pages = p->n_pages;
    a.nb = su.nb; a.m_cap = su.m_cap; a.wide = su.wide ? 1 : 0;
    a.seg_tiles = kSegTiles;
    a.cost_base = cost_base_for(*p, su);
    a.plan = nullptr; a.plan_key = 0;
}

// All attention entry points.  kv8: the caches hold E4M3 bytes with per-head scales (stream kernel only).
// plan: schedule built by fsr_attn_plan for the same shapes and device arrays, or null.
int attention_call(const void* q, const void* k_cache, const void* v_cache, const float* k_scale, const float* v_scale, bool kv8,
                   const int32_t* block_tables, const int32_t* ctx_lens, const int32_t* cu_q, void* out, float* lse,
                   const fsr_attn_params* p, const void* plan, void* workspace, size_t ws_bytes, int shares_cap, void* stream,
                   const char* who) {
    int rc = validate(p, who);
    if (rc != FSR_OK) return rc;
    if (p->B == 0 || p->N_cap == 0) return FSR_OK;
    if (!q || !k_cache || !v_cache || !block_tables || !ctx_lens || !cu_q || !out)
        return fail(FSR_EINVAL, "%s: null pointer among q/k_cache/v_cache/block_tables/ctx_lens/cu_q/out", who);
    if (kv8 && (!k_scale || !v_scale)) return fail(FSR_EINVAL, "%s: k_scale / v_scale is null", who);
    hipStream_t s = (hipStream_t)stream;
    const Setup su = make_setup(*p, shares_cap);
    if (kv8 && !su.fast)
        return fail(FSR_EUNSUP, "%s: 8-bit caches need bf16 queries, D = 128, P = 16, H_q / H_kv <= 16, B <= %d", who, kMaxB);
    if (plan && !su.fast)
        return fail(FSR_EUNSUP, "%s: a plan needs the stream kernel (bf16, D = 128, P = 16, H_q / H_kv <= 16, B <= %d)", who, kMaxB);
    if (su.fast) {
        const size_t need = su.ws_bytes();
        if (!workspace || ws_bytes < need) return fail(FSR_EWS, "%s: workspace %zu bytes, need %zu", who, ws_bytes, need);
        if ((uintptr_t)workspace & 255) return fail(FSR_EWS, "%s: workspace must be 256-byte aligned", who);
        if (((uintptr_t)q | (uintptr_t)k_cache | (uintptr_t)v_cache | (uintptr_t)out) & 15)
            return fail(FSR_EINVAL, "%s: q/k_cache/v_cache/out must be 16-byte aligned", who);
        FastArgs a;
        fill_common(a, p, su, block_tables, ctx_lens, cu_q);
        a.q = (const uint16_t*)q; a.k = (const uint16_t*)k_cache; a.v = (const uint16_t*)v_cache;
        a.out = out; a.lse = lse;
        a.part_o = (float*)workspace;
        a.part_ml = (float*)((char*)workspace + su.bytes_o);
        a.arrivals = (unsigned long long*)((char*)workspace + su.bytes_o + su.bytes_ml);
        a.call_id = next_call_id();
        a.out_bf16 = p->out_dtype == FSR_BF16;
        a.scale_log2 = p->scale * kLog2e;
        a.k_scale = k_scale; a.v_scale = v_scale;
        if (plan) {
            const uint32_t key = plan_key_of(*p, su);
            {
                std::lock_guard<std::mutex> lock(g_plans_mutex);
                const auto it = g_plans.find(plan);
                if (it == g_plans.end()) return fail(FSR_EINVAL, "%s: no plan has been built in this buffer (fsr_attn_plan)", who);
                if (it->second != key)
                    return fail(FSR_ESHAPE, "%s: the plan was built for other shapes (B, N_cap, heads, max_pages, n_pages, max_q_len, max_workgroups)", who);
            }
            if ((uintptr_t)plan & 15) return fail(FSR_EINVAL, "%s: plan must be 16-byte aligned", who);
            a.plan = (const int32_t*)plan;
            a.plan_key = key;
        }
        const dim3 grid(su.nb), block(kThreads);
        const size_t smem = plan ? planned_smem(su.mt_max, su.wide) : stream_fixed_smem(su.wide) + tables_bytes(p->B);
#define FSR_LAUNCH_K(KERNEL, MT, WIDE)                                                       \
    if (kv8 && p->kv_layout == FSR_KV_TOKEN_MAJOR)                                           \
        hipLaunchKernelGGL((KERNEL<MT, true, true, WIDE>), grid, block, smem, s, a);         \
    else if (kv8)                                                                            \
        hipLaunchKernelGGL((KERNEL<MT, false, true, WIDE>), grid, block, smem, s, a);        \
    else if (p->kv_layout == FSR_KV_TOKEN_MAJOR)                                             \
        hipLaunchKernelGGL((KERNEL<MT, true, false, WIDE>), grid, block, smem, s, a);        \
    else                                                                                     \
        hipLaunchKernelGGL((KERNEL<MT, false, false, WIDE>), grid, block, smem, s, a)
#define FSR_LAUNCH(MT, WIDE)                                    \
    if (plan) { FSR_LAUNCH_K(attn_planned_kernel, MT, WIDE); }  \
    else { FSR_LAUNCH_K(attn_stream_kernel, MT, WIDE); }
        if (su.wide) {
            FSR_LAUNCH(kWideMT, true);
        } else {
            switch (su.mt_max) {
                case 1: FSR_LAUNCH(1, false); break;
                case 2: FSR_LAUNCH(2, false); break;
                case 3: FSR_LAUNCH(3, false); break;
                default: FSR_LAUNCH(4, false); break;
            }
        }
#undef FSR_LAUNCH
#undef FSR_LAUNCH_K
        return check_launch(plan ? "attn_planned_kernel" : "attn_stream_kernel");
    }
    GenericArgs g;
    g.q = q; g.k = k_cache; g.v = v_cache; g.bt = block_tables; g.ctx = ctx_lens; g.cu_q = cu_q; g.out = out; g.lse = lse;
    g.B = p->B; g.H_q = p->H_q; g.H_kv = p->H_kv; g.P = p->P; g.max_pages = p->max_pages; g.n_pages = p->n_pages;
    g.scale = p->scale;
    g.token_major = p->kv_layout == FSR_KV_TOKEN_MAJOR;
    const dim3 grid(p->H_q, p->N_cap), block(64);
    if (p->N_cap > 65535) return fail(FSR_EUNSUP, "%s: the one-wave-per-row path is limited to N_cap <= 65535 rows", who);
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
}  // namespace

extern "C" int fsr_verify_attention(const void* q, const void* k_cache, const void* v_cache,
                                    const int32_t* block_tables, const int32_t* ctx_lens, const int32_t* spec_lens,
                                    const int32_t* cu_q, void* out, float* lse, const fsr_attn_params* p,
                                    void* workspace, size_t ws_bytes, void* stream) {
    (void)spec_lens;
    return attention_call(q, k_cache, v_cache, nullptr, nullptr, false, block_tables, ctx_lens, cu_q, out, lse, p, nullptr, workspace,
                          ws_bytes, kMaxShares, stream, "fsr_verify_attention");
}

extern "C" int fsr_verify_attention_kv8(const void* q, const void* k_cache, const void* v_cache, const float* k_scale,
                                        const float* v_scale, const int32_t* block_tables, const int32_t* ctx_lens,
                                        const int32_t* cu_q, void* out, float* lse, const fsr_attn_params* p,
                                        void* workspace, size_t ws_bytes, void* stream) {
    return attention_call(q, k_cache, v_cache, k_scale, v_scale, true, block_tables, ctx_lens, cu_q, out, lse, p, nullptr, workspace,
                          ws_bytes, kMaxShares, stream, "fsr_verify_attention_kv8");
}

extern "C" int fsr_attn_plan(const int32_t* block_tables, const int32_t* ctx_lens, const int32_t* cu_q,
                             const fsr_attn_params* p, void* plan, size_t plan_bytes, void* stream) {
    int rc = validate(p, "fsr_attn_plan");
    if (rc != FSR_OK) return rc;
    if (!block_tables || !ctx_lens || !cu_q || !plan) return fail(FSR_EINVAL, "fsr_attn_plan: null pointer among block_tables/ctx_lens/cu_q/plan");
    const Setup su = make_setup(*p);
    if (!su.fast)
        return fail(FSR_EUNSUP, "fsr_attn_plan: only the stream kernel takes a plan (bf16, D = 128, P = 16, H_q / H_kv <= 16, B <= %d)", kMaxB);
    const size_t need = plan_bytes_of(*p, su);
    if (plan_bytes < need) return fail(FSR_EWS, "fsr_attn_plan: plan buffer %zu bytes, need %zu", plan_bytes, need);
    if ((uintptr_t)plan & 15) return fail(FSR_EINVAL, "fsr_attn_plan: plan must be 16-byte aligned");
    FastArgs a{};
    fill_common(a, p, su, block_tables, ctx_lens, cu_q);
    a.plan_key = plan_key_of(*p, su);
    const size_t smem = tables_bytes(p->B) + (size_t)kMaxShares * sizeof(int);
    hipLaunchKernelGGL(attn_plan_kernel, dim3(1), dim3(kThreads), smem, (hipStream_t)stream, a, su.mt_max, (int32_t*)plan,
                       (int)plan_more_cap(*p, su));
    rc = check_launch("attn_plan_kernel");
    if (rc == FSR_OK) {
        std::lock_guard<std::mutex> lock(g_plans_mutex);
        g_plans[plan] = a.plan_key;
    }
    return rc;
}

extern "C" int fsr_verify_attention_planned(const void* q, const void* k_cache, const void* v_cache,
                                            const int32_t* block_tables, const int32_t* ctx_lens, const int32_t* cu_q,
                                            void* out, float* lse, const fsr_attn_params* p, const void* plan,
                                            void* workspace, size_t ws_bytes, void* stream) {
    if (!plan) return fail(FSR_EINVAL, "fsr_verify_attention_planned: plan is null");
    return attention_call(q, k_cache, v_cache, nullptr, nullptr, false, block_tables, ctx_lens, cu_q, out, lse, p, plan, workspace,
                          ws_bytes, kMaxShares, stream, "fsr_verify_attention_planned");
}

extern "C" int fsr_verify_attention_kv8_planned(const void* q, const void* k_cache, const void* v_cache, const float* k_scale,
                                                const float* v_scale, const int32_t* block_tables, const int32_t* ctx_lens,
                                                const int32_t* cu_q, void* out, float* lse, const fsr_attn_params* p,
                                                const void* plan, void* workspace, size_t ws_bytes, void* stream) {
    if (!plan) return fail(FSR_EINVAL, "fsr_verify_attention_kv8_planned: plan is null");
    return attention_call(q, k_cache, v_cache, k_scale, v_scale, true, block_tables, ctx_lens, cu_q, out, lse, p, plan, workspace,
                          ws_bytes, kMaxShares, stream, "fsr_verify_attention_kv8_planned");
}

// ---------------------------------------------------------------------------------------
// fsr_verify_attention_static: the same call for callers that cannot allocate (or be handed) a
// workspace.  The partial slots and arrival words live in a file-scope device array, laid out for
// kStaticShares workgroups (MI355X has 256 compute units; a device with more runs a 256-workgroup
// grid here).  Every GPU holds its own copy of the array at its own address, looked up once per
// device; all calls on a GPU share it, so calls that overlap in time on one GPU race.
// ---------------------------------------------------------------------------------------
namespace {
constexpr int kStaticShares = 256;
constexpr size_t kStaticScratchBytes =
    (size_t)kStaticShares * 2 * 16 * 2 * kWideMT * (kD + 4) * sizeof(float) + (size_t)(kStaticShares + 1) * sizeof(unsigned long long) + 3 * 256;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {nullptr};

// Device address of `scratch` on the current device (0 on failure, with the error text set).
void* static_scratch() {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) {
        fail(FSR_EHIP, "fsr_verify_attention_static: hipGetDevice: %s", hipGetErrorString(e));
        return nullptr;
    }
    if (dev < 0 || dev >= kMaxDevices) {
        fail(FSR_EUNSUP, "fsr_verify_attention_static: device index %d (at most %d devices)", dev, kMaxDevices);
        return nullptr;
    }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr) {
            fail(FSR_EHIP, "fsr_verify_attention_static: hipGetSymbolAddress: %s", hipGetErrorString(e));
            return nullptr;
        }
        g_scratch_ptr[dev] = ptr;
    }
    return g_scratch_ptr[dev];
}
}  // namespace

extern "C" size_t fsr_static_scratch_bytes(void) { return kStaticScratchBytes; }

extern "C" int fsr_verify_attention_static(const void* q, const void* k_cache, const void* v_cache,
                                           const int32_t* block_tables, const int32_t* ctx_lens, const int32_t* cu_q,
                                           void* out, float* lse, const fsr_attn_params* p, void* stream) {
    int rc = validate(p, "fsr_verify_attention_static");
    if (rc != FSR_OK) return rc;
    const Setup su = make_setup(*p, kStaticShares);
    if (!su.fast)  // the one-wave-per-row kernel uses no scratch buffer at all
        return attention_call(q, k_cache, v_cache, nullptr, nullptr, false, block_tables, ctx_lens, cu_q, out, lse, p, nullptr, nullptr, 0,
                              kStaticShares, stream, "fsr_verify_attention_static");
    if (su.ws_bytes() > kStaticScratchBytes)
        return fail(FSR_EWS, "fsr_verify_attention_static: these shapes need %zu bytes of scratch, the built-in buffer has %zu",
                    su.ws_bytes(), kStaticScratchBytes);
    void* ws = static_scratch();
    if (!ws) return FSR_EHIP;
    return attention_call(q, k_cache, v_cache, nullptr, nullptr, false, block_tables, ctx_lens, cu_q, out, lse, p, nullptr, ws,
                          kStaticScratchBytes, kStaticShares, stream, "fsr_verify_attention_static");
}
