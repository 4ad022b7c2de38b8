// libkb: C ABI, host-side planning, and the small kernels around the scan (gfx950 only).
//
//   kb_normalize : row_norm_kernel            (row L2 norms as a side scale)
//   kb_query     : scan kernel, sampling pass (kb_scan.hpp)
//                  threshold_kernel           (k-th best group maximum per query; query norms, counters reset)
//                  [prep_kernel               (query norms, counters reset: when no sampling pass runs)]
//                  scan kernel, main pass     (kb_scan.hpp; its wavefronts move their records to per-query lists)
//                  finalize_kernel            (top k of each query's list by radix selection; or the
//                                              exhaustive per-query scan when a list overflowed)
#include <stdlib.h>
#include <string.h>

#include <new>

#include "kb_configs.hpp"
#include "kb_internal.hpp"
#include "kb_scan.hpp"

using namespace kbi;


namespace kbi {

thread_local ScanTiming scan_timing;

bool scan_config_info(int key_dtype, int config, ConfigInfo *out)
{
#define X(ID, KT, TK, TQ, WM, WN, RBA, NSTAGE, WGPC)                          \
    if (key_dtype == KT && config == ID) {                                    \
        *out = ConfigInfo{TK, TQ, 64 * WM * WN, WM * 2, WGPC, RBA, 0};    \
        return true;                                                          \
    }
    KB_SCAN_CONFIGS_BF16(X)
    KB_SCAN_CONFIGS_F32(X)
    KB_SCAN_CONFIGS_FP8(X)
#undef X
#define X(ID, KT, TK, TQ, WM, WN, RBA, NSTAGE, WGPC)                          \
    if (key_dtype == KB_FP8_E4M3 && config == ID) {                           \
        *out = ConfigInfo{TK, TQ, 64 * WM * WN, WM * 2, WGPC, RBA, 0};    \
        return true;                                                          \
    }
    KB_SCAN_CONFIGS_FP8_Q8(X)
#undef X
#define XS(ID, KT, TQ, NSA, NSB)                                              \
    if (key_dtype == KT && config == ID) {                                    \
        *out = ConfigInfo{256, TQ, 512, 8, 1, 64 * ((NSA > NSB ? NSA : NSB) + 1), 3}; \
        return true;                                                          \
    }
    KB_SCAN_SP_CONFIGS_BF16_IL(XS)
    KB_SCAN_SP_CONFIGS_FP8(XS)
    KB_SCAN_SP_CONFIGS_FP8_Q8(XS)
#undef XS
#define XW(ID, KT, TQ)                                                        \
    if (key_dtype == KT && config == ID) {                                    \
        *out = ConfigInfo{256, TQ, 512, 8, 1, 512, 4};                        \
        return true;                                                          \
    }
    KB_SCAN_WIDE_CONFIGS_BF16(XW)
    KB_SCAN_WIDE_CONFIGS_FP8_Q8(XW)
#undef XW
    return false;
}

constexpr int64_t WIDE128_MIN_ROWS = 4 * 65536;     // rows from which the 128-query full-line kernel is the faster one (measured: 2^18)

int scan_config_for(int key_dtype, int Q, int d, int64_t n)
{
    if (key_dtype == KB_BF16 && Q > 128 && d * 2 >= 512) return 18;
    // 33 to 128 queries: the full-line kernel once a workgroup has several tiles to stream (its ring takes longer to fill)
    if (key_dtype == KB_BF16 && Q > 32 && d * 2 >= 512 && n >= WIDE128_MIN_ROWS) return 19;
    if (key_dtype == KB_BF16 && Q > 128 && d * 2 >= 384) return 17;
    if (key_dtype == KB_FP8_E4M3 && Q > 128 && d >= 256) return 4;
    // below that size a query is bound by the latency of its launches: tiles of 64 rows (twice the workgroups, half the
    // chunks each) finish sooner: 62 against 71 us per call on 65,536 rows of 768 bf16 values with 64 queries
    // (and 64 against 70 us with 128 queries)
    if (key_dtype == KB_BF16 && Q > 32 && Q <= 128 && n < WIDE128_MIN_ROWS) return Q <= 64 ? 12 : 16;
    return Q <= 32 ? 1 : Q <= 128 ? 2 : 3;
}

}  // namespace kbi

namespace {

constexpr int DEVICE_CUS = 256;        // compute units of an MI355X: the scan grids are sized for them (a device with fewer runs the same grid in turns)
constexpr int MAX_REGION_CAP = 8192;   // records a scan wavefront collects at most before it moves them to the lists
constexpr int MAX_SAMPLE_SLOTS = 8192; // threshold_kernel sorts this many 64-bit words in LDS (64 KiB)
constexpr int MAX_CAND_CAP = 8192;     // finalize_kernel likewise
constexpr int MIN_CAND_CAP = 1024;
constexpr int FALLBACK_PARTS = 32;    // workgroups that share the rows of a query on the exhaustive path
constexpr size_t WS_ALIGN = 256;
constexpr int FP8_QUERY_CONFIG = 5;    // scan configuration of fp8 keys with fp8 queries (kb_configs.hpp)
constexpr int FP8_QUERY_WIDE_CONFIG = 20;     // ... with 128-byte row pieces: rows of a multiple of 128 bytes, 512 at least
constexpr int FP8_QUERY_TILED_CONFIG = 6;     // ... the tiled kernel: 6, 7, 8 for query blocks of 64, 128, 256; every row length
bool is_fp8_query_config(int config)
{
    return config == FP8_QUERY_CONFIG || config == FP8_QUERY_WIDE_CONFIG || (config >= FP8_QUERY_TILED_CONFIG && config <= FP8_QUERY_TILED_CONFIG + 2);
}

int key_bytes(kb_dtype_t t) { return t == KB_F32 ? 4 : t == KB_BF16 ? 2 : 1; }
int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
int64_t pow2_ceil(int64_t x)
{
    int64_t p = 1;
    while (p < x) p <<= 1;
    return p;
}
size_t align_up(size_t x) { return (x + WS_ALIGN - 1) / WS_ALIGN * WS_ALIGN; }

// Multiplier of the sampling pass's scatter j -> (j * m) mod n over the n runs of rows: about n / golden ratio, so
// that consecutive j land far apart and fill the range evenly, and coprime to n, so that the map is one to one.
// 0 (no scatter) when there are too few runs.
uint64_t scatter_multiplier(int64_t n)
{
    if (n < 3) return 0;
    uint64_t m = (uint64_t)((double)n * 0.6180339887498949) | 1u;
    for (;; m += 2) {
        uint64_t a = m, b = (uint64_t)n;
        while (b) {
            const uint64_t t = a % b;
            a = b;
            b = t;
        }
        if (a == 1) return m % (uint64_t)n;
    }
}

// ------------------------------------------------------------------------------------------------
// Planning: which kernels a query runs, how large its buffers are, where they live in the workspace.
// ------------------------------------------------------------------------------------------------
struct Choice {                 // kernels of a query over n rows
    int config;
    ConfigInfo ci;
    int sample_config;          // the sampling pass may run another configuration (same tile, bit-identical scores)
    ConfigInfo sci;
};

bool choose_kernels(const kb *h, int64_t n, int32_t Q, bool draw, bool q8, Choice *out)
{
    Choice c;
    const int generic = Q <= 32 ? 1 : Q <= 128 ? 2 : 3;        // the tiled kernel: every dtype, every row length
    const size_t row_bytes = (size_t)h->d * key_bytes(h->dtype);
    if (q8) {       // fp8 queries: only the kernels built on the fp8 matrix instruction take them
        if (h->dtype != KB_FP8_E4M3) return false;
        const int generic8 = Q <= 64 ? FP8_QUERY_TILED_CONFIG : Q <= 128 ? FP8_QUERY_TILED_CONFIG + 1 : FP8_QUERY_TILED_CONFIG + 2;
        // large batches: the pipelined kernels (256-query blocks); smaller ones would pad their query columns there
        c.config = Q <= 128 ? generic8 : (row_bytes % 128 == 0 && row_bytes >= 512) ? FP8_QUERY_WIDE_CONFIG : FP8_QUERY_CONFIG;
        if (is_fp8_query_config((int)h->tune_config)) c.config = (int)h->tune_config;         // another one can be asked for
        if (!scan_config_info(h->dtype, c.config, &c.ci)) return false;
        // the weighted random selection exists in the tiled kernel only, and rows may be too short for a pipelined kernel
        if ((draw && c.ci.family != 0) || row_bytes < (size_t)c.ci.min_row_bytes) {
            c.config = generic8;
            if (!scan_config_info(h->dtype, c.config, &c.ci)) return false;
        }
    } else {
        c.config = h->tune_config > 0 ? (int)h->tune_config : scan_config_for(h->dtype, Q, h->d, n);
        if (!scan_config_info(h->dtype, c.config, &c.ci)) return false;
        // fall back where a (forced) configuration does not apply: the weighted random selection exists in the
        // tiled kernel and in the main pass of the bf16 full-line kernel, rows may be too short for a pipelined kernel,
        // and the fp8-query kernels read fp8 queries
        const bool draws = c.ci.family == 0 || (c.ci.family == 4 && h->dtype == KB_BF16);
        if ((draw && !draws) || row_bytes < (size_t)c.ci.min_row_bytes || (h->dtype == KB_FP8_E4M3 && is_fp8_query_config(c.config))) {
            c.config = generic;
            if (!scan_config_info(h->dtype, c.config, &c.ci)) return false;
        }
    }
    c.sci = c.ci;
    c.sample_config = c.config;
    if (c.ci.family == 4 && h->dtype == KB_FP8_E4M3) {       // the fp8 full-line kernel is a main pass only
        c.sample_config = FP8_QUERY_CONFIG;
        if (!scan_config_info(h->dtype, c.sample_config, &c.sci) || c.sci.tq != c.ci.tq || c.sci.tk != c.ci.tk) return false;
    }
    if (draw && c.ci.family == 4) {     // so is the full-line kernel on keys: the tiled kernel with the same query blocks samples
        c.sample_config = c.ci.tq == 128 ? 2 : 3;
        if (!scan_config_info(h->dtype, c.sample_config, &c.sci) || c.sci.tq != c.ci.tq || c.sci.family != 0) return false;
    }
    *out = c;
    return true;
}

// Key tiles the sampling pass scores when the knowledge base has nt tiles: max(k, 8) / 512 of them (1/64 of the
// rows up to k = 8, 1/16 at k = 32, 1/4 at k = 128), at least two samples per wanted result, at most what the
// threshold kernel sorts and half of the tiles.  A sampling pass of few tiles is bound by the latency of one tile, not
// by its bytes: as long as the sample stays small (FREE_SAMPLE_BYTES of keys, a quarter of the tiles) it takes as many
// tiles as the device runs side by side, which costs no time and thins the candidates of the main pass.
// 0 = no sampling pass (every entry is a candidate).  Depends on the row count through nt only, and never falls as
// nt grows (`floor` switched off).
constexpr int64_t FREE_SAMPLE_BYTES = 32 << 20;
int64_t sample_tiles_for(const kb *h, const ConfigInfo &sci, int64_t nt, int32_t Q, int32_t k, bool floor)
{
    if (nt < 8) return 0;
    const int64_t kk = k > 8 ? k : 8;
    int64_t st = h->tune_sample_keys > 0 ? ceil_div(h->tune_sample_keys, sci.tk) : ceil_div(nt * kk, 512);
    const int64_t want = ceil_div(2 * (int64_t)k, sci.groups_per_tile);
    if (st < want) st = want;
    if (h->tune_sample_keys <= 0) {
        const int64_t nqb = ceil_div(Q, sci.tq);
        int64_t free_tiles = (int64_t)DEVICE_CUS * sci.wg_per_cu / nqb;
        const int64_t by_bytes = FREE_SAMPLE_BYTES / ((int64_t)sci.tk * h->d * key_bytes(h->dtype));
        if (free_tiles > by_bytes) free_tiles = by_bytes;
        if (free_tiles > nt / 4) free_tiles = nt / 4;
        if (st < free_tiles) st = free_tiles;
    }
    if (st > MAX_SAMPLE_SLOTS / sci.groups_per_tile) st = MAX_SAMPLE_SLOTS / sci.groups_per_tile;
    if (st > nt / 2) st = nt / 2;
    if (floor && st * sci.groups_per_tile < k) st = 0;
    return st;
}

int32_t cand_cap_for(int64_t expect, bool sampled)
{
    int64_t cc = pow2_ceil(sampled ? 8 * expect : expect);
    if (cc < MIN_CAND_CAP) cc = MIN_CAND_CAP;
    if (cc > MAX_CAND_CAP) cc = MAX_CAND_CAP;
    return (int32_t)cc;
}

// Sizes of the workspace arrays.  The layout is a function of these alone and its total grows with each of them.
struct Sizes {
    int32_t k, qpad, regions, sample_slots, cand_cap;
    int64_t region_records;     // scan wavefronts * region_cap
    int64_t lgain_rows;
};

void lay_out(const Sizes &z, Plan *p)
{
    size_t off = 0;
    p->off_stats = off;       off = align_up(off + sizeof(uint64_t) * (STAT_WORDS + STAT_PARTIALS));   // always first: kb_query_counters reads it
    p->off_invq = off;        off = align_up(off + sizeof(float) * z.qpad);
    p->off_thr64 = off;       off = align_up(off + sizeof(uint64_t) * z.qpad);
    p->off_thrp = off;        off = align_up(off + sizeof(float) * z.qpad);
    p->off_cnt = off;         off = align_up(off + sizeof(uint32_t) * z.qpad * CAND_SEGMENTS);
    p->off_flag = off;        off = align_up(off + sizeof(uint32_t) * z.qpad);
    p->fb_parts = z.cand_cap / KB_K_MAX < FALLBACK_PARTS ? z.cand_cap / KB_K_MAX : FALLBACK_PARTS;     // parts * k words fit the LDS buffer
    p->off_fb_done = off;     off = align_up(off + sizeof(uint32_t) * z.qpad);
    p->off_fb_lists = off;    off = align_up(off + sizeof(uint64_t) * (size_t)z.qpad * p->fb_parts * z.k);
    p->off_qmask = off;       off = align_up(off + sizeof(uint64_t) * z.qpad);
    p->off_samp = off;        off = align_up(off + sizeof(uint64_t) * (size_t)z.qpad * (z.sample_slots > 0 ? z.sample_slots : 1));
    p->off_regions = off;     off = align_up(off + sizeof(Record) * (size_t)z.region_records);
    p->off_cand = off;        off = align_up(off + sizeof(uint64_t) * (size_t)z.qpad * z.cand_cap);
    p->off_lgain = off;       off = align_up(off + sizeof(float) * (size_t)z.lgain_rows);   // ln(gain), padded past the last tile
    p->total = off;
}

// The plan of a query over n rows with the kernels `c`.  Apart from the ln(gain) array it depends on n through the
// number of key tiles only, which is what lets kb_query_workspace_bytes bound it over all row counts.
void plan_for(const kb *h, const Choice &c, int64_t n, int32_t Q, int32_t k, bool draw, Plan *out, Sizes *sizes)
{
    Plan p;
    memset(&p, 0, sizeof p);
    const ConfigInfo &ci = c.ci, &sci = c.sci;
    p.Q = Q;
    p.k = k;
    p.config = c.config;
    p.family = ci.family;
    p.tk = ci.tk;
    p.tq = ci.tq;
    p.groups_per_tile = ci.groups_per_tile;
    p.nqb = (int32_t)ceil_div(Q, ci.tq);
    p.qpad = p.nqb * ci.tq;
    p.sample_config = c.sample_config;
    p.sample_family = sci.family;
    p.sample_wgpc = sci.wg_per_cu;
    if (n < 1) n = 1;
    const int64_t nt = ceil_div(n, ci.tk), nts = ceil_div(n, sci.tk);     // key tiles of the main pass, of the sampling pass

    const int64_t st = sample_tiles_for(h, sci, nts, Q, k, true);
    p.sample_tk = sci.tk;
    p.sample_tiles = st;
    p.sample_slots = (int32_t)(st * sci.groups_per_tile);
    p.sample_keys = st * sci.tk;
    const int64_t expect = st > 0 ? ceil_div((int64_t)k * nts, st) : nt * ci.tk;      // candidates per query
    p.cand_cap = cand_cap_for(expect, st > 0);

    const int wgpc = h->tune_wg_per_cu > 0 ? (int)h->tune_wg_per_cu : ci.wg_per_cu;
    const int64_t items = nt * p.nqb;
    const int64_t grid = items < (int64_t)DEVICE_CUS * wgpc ? items : (int64_t)DEVICE_CUS * wgpc;
    p.grid = (int32_t)grid;
    const int waves = ci.threads / 64;
    p.regions = (int32_t)(grid * waves);
    // Records a scan wavefront collects before it moves them to the per-query lists.  With a sampling pass few pairs
    // pass the filter (a wavefront sees some tens in a whole scan).  Without one every scored pair is a record: room
    // for the pairs of the wavefront's part of its workgroup's items, within limits.
    int64_t rc = REGION_CAP;
    if (st == 0) {
        rc = pow2_ceil(ceil_div(items, grid) * ci.tk * ci.tq / waves);
        if (rc < REGION_CAP) rc = REGION_CAP;
        if (rc > MAX_REGION_CAP) rc = MAX_REGION_CAP;
    }
    p.region_cap = (int32_t)rc;

    Sizes z;
    z.k = k;
    z.qpad = p.qpad;
    z.regions = p.regions;
    z.sample_slots = p.sample_slots;
    z.cand_cap = p.cand_cap;
    z.region_records = (int64_t)p.regions * rc;
    z.lgain_rows = draw ? ceil_div(n, 256) * 256 + 256 : 0;      // the weighted random selection only
    lay_out(z, &p);
    *out = p;
    if (sizes) *sizes = z;
}

// Pure function of (handle settings, row count n, Q, k): which kernels run on what, and where everything lives
// in the workspace.
bool make_plan(const kb *h, int64_t n, int32_t Q, int32_t k, bool draw, bool q8, Plan *out)
{
    Choice c;
    if (!choose_kernels(h, n, Q, draw, q8, &c)) return false;
    plan_for(h, c, n, Q, k, draw, out, nullptr);
    return true;
}

void max_into(Sizes &m, const Sizes &z)
{
    m.k = z.k;
    if (z.qpad > m.qpad) m.qpad = z.qpad;
    if (z.regions > m.regions) m.regions = z.regions;
    if (z.sample_slots > m.sample_slots) m.sample_slots = z.sample_slots;
    if (z.cand_cap > m.cand_cap) m.cand_cap = z.cand_cap;
    if (z.region_records > m.region_records) m.region_records = z.region_records;
    if (z.lgain_rows > m.lgain_rows) m.lgain_rows = z.lgain_rows;
}

// Upper bound of the Sizes of plan_for(h, c, n, ...) over every n in [1, capacity].  nt counts the key tiles of the
// sampling configuration (its tiles may be lower than the main pass's; both counts are constant between multiples of
// the lower tile height).
//   Up to EXACT_TILES key tiles the plans are enumerated (one per pair of tile counts; this range contains every case
//   without a sampling pass: sample_tiles_for gives at least min(2k / groups, nt / 2) tiles, which is k samples once
//   nt >= 256).
//   Beyond, with st = sample_tiles_for(nt) > 0 and expect = ceil(k nt / st):
//     st = ceil(nt max(k, 8) / 512), or raised to 2k / groups:  expect <= 512
//     st = nt / 2 (rounded down):                               expect <= 2k + 1 <= 257
//     st = MAX_SAMPLE_SLOTS / groups:                           expect grows with nt, largest at the capacity
//   (with the "sample_keys" knob st does not follow nt: the largest candidate capacity is assumed), so cand_cap is
//   bounded; the number of scan wavefronts and sample_slots do not fall as nt grows, and region_cap is REGION_CAP.
constexpr int64_t EXACT_TILES = 256;
void bound_sizes(const kb *h, const Choice &c, int32_t Q, int32_t k, bool draw, Sizes &m)
{
    const ConfigInfo &ci = c.ci, &sci = c.sci;
    const int64_t step = ci.tk < sci.tk ? ci.tk : sci.tk;
    const int64_t cap_nt = ceil_div(h->capacity, sci.tk);
    Plan p;
    Sizes z;
    for (int64_t n = step; n < h->capacity + step && ceil_div(n, sci.tk) <= EXACT_TILES; n += step) {
        plan_for(h, c, n, Q, k, draw, &p, &z);
        max_into(m, z);
    }
    plan_for(h, c, h->capacity, Q, k, draw, &p, &z);       // the ln(gain) array, and the largest grid
    max_into(m, z);
    if (cap_nt <= EXACT_TILES) return;
    int64_t expect = 512;
    const int64_t at_cap = ceil_div((int64_t)k * cap_nt * sci.groups_per_tile, MAX_SAMPLE_SLOTS);
    if (at_cap > expect) expect = at_cap;
    z.cand_cap = h->tune_sample_keys > 0 ? MAX_CAND_CAP : cand_cap_for(expect, true);
    z.sample_slots = (int32_t)(sample_tiles_for(h, sci, cap_nt, Q, k, false) * sci.groups_per_tile);
    z.region_records = (int64_t)z.regions * REGION_CAP;
    max_into(m, z);
}

// ------------------------------------------------------------------------------------------------
// row norms
// ------------------------------------------------------------------------------------------------
template <int DT> __device__ inline float piece_sum_squares(u32x4 v);
template <> __device__ inline float piece_sum_squares<KB_F32>(u32x4 v)
{
    float s = 0.f;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const float x = as_f32(v[e]);
        s += x * x;
    }
    return s;
}
template <> __device__ inline float piece_sum_squares<KB_BF16>(u32x4 v)
{
    float s = 0.f;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const float lo = as_f32(v[e] << 16), hi = as_f32(v[e] & 0xffff0000u);
        s += lo * lo;
        s += hi * hi;
    }
    return s;
}
template <> __device__ inline float piece_sum_squares<KB_FP8_E4M3>(u32x4 v)
{
    float s = 0.f;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const f32x2 a = __builtin_amdgcn_cvt_pk_f32_fp8(v[e], false), b = __builtin_amdgcn_cvt_pk_f32_fp8(v[e], true);
        s += a.x * a.x;
        s += a.y * a.y;
        s += b.x * b.x;
        s += b.y * b.y;
    }
    return s;
}

__device__ inline float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// One wavefront per row: lanes stride over the row's 16-byte pieces, fp32 sum of squares, butterfly
// reduction, inv = 1/sqrt(sum) or 0 for a zero row.
template <int DT> __device__ inline float row_inv_norm(const void *base, int64_t row, int row_bytes, int lane)
{
    const u32x4 *p = reinterpret_cast<const u32x4 *>(static_cast<const unsigned char *>(base) + (size_t)row * row_bytes);
    float s = 0.f;
    for (int i = lane; i < row_bytes / 16; i += 64) s += piece_sum_squares<DT>(__builtin_nontemporal_load(p + i));
    s = wave_sum(s);
    return s > 0.f ? 1.0f / sqrtf(s) : 0.f;
}

template <int DT> __global__ __launch_bounds__(256) void row_norm_kernel(const void *keys, int64_t begin, int64_t end, int d, float *inv_norm)
{
    const int lane = threadIdx.x & 63;
    const int64_t row = begin + (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= end) return;
    const float inv = row_inv_norm<DT>(keys, row, d * (DT == KB_F32 ? 4 : DT == KB_BF16 ? 2 : 1), lane);
    if (lane == 0) inv_norm[row] = inv;
}

// ------------------------------------------------------------------------------------------------
// weighted random selection: ln(gain) per entry, -inf for entries without weight and for the padding
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void log_gain_kernel(const float *gain, int64_t n, int64_t n_padded, float *log_gain)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n_padded) return;
    float v = -__builtin_inff();
    if (i < n) {
        const float g = gain[i];
        if (g > 0.f) v = logf(g);
    }
    log_gain[i] = v;
}

// ------------------------------------------------------------------------------------------------
// prep: query norms + reset of the per-call counters
// ------------------------------------------------------------------------------------------------
template <int QT> __global__ __launch_bounds__(256) void prep_kernel(const void *queries, int Q, int qpad, int d, float *invq, uint64_t *thr64, float *thrp,
                                                                       uint32_t *cnt, uint32_t *flag, uint64_t *stats, uint64_t sample_keys,
                                                                       const uint64_t *qmask, uint64_t *qmask_pad, int grid, uint32_t *fb_done)
{
    const int t = blockIdx.x * 256 + threadIdx.x;
    if (t < qpad) fb_done[t] = 0;
    if (t < qpad) {     // padding queries (t >= Q) can never pass the filter of the scan
        thr64[t] = t < Q ? 0ull : ~0ull;
        thrp[t] = t < Q ? -__builtin_inff() : __builtin_inff();
        for (int sg = 0; sg < CAND_SEGMENTS; ++sg) cnt[t * CAND_SEGMENTS + sg] = 0;
        flag[t] = 0;
        qmask_pad[t] = (qmask && t < Q) ? qmask[t] : 0ull;
    }
    if (t < STAT_WORDS + STAT_PARTIALS) stats[t] = t == 2 ? sample_keys : t == 3 ? (uint64_t)grid : 0ull;
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row < qpad) {
        const float inv = row < Q ? row_inv_norm<QT>(queries, row, d * (QT == KB_F32 ? 4 : QT == KB_BF16 ? 2 : 1), lane) : 0.f;
        if (lane == 0) invq[row] = inv;
    }
}

// ------------------------------------------------------------------------------------------------
// A full sort is a chain of dependent LDS round trips (one per stage) and costs tens of microseconds for a
// few thousand words.  Selection needs far fewer: a most-significant-digit radix search for the k-th
// largest word (8-bit digits, starting at the highest bit in which the words' upper halves differ; each pass is
// one histogram with LDS atomics and one wavefront-wide scan), then the survivors are compacted
// and ordered by counting, for each, how many survivors are larger.  The selection runs in kernels whose whole
// length is a few microseconds, so its own fixed costs count: the reductions and scans across lanes are
// data-parallel-primitive moves (a shuffle is an LDS round trip each), the wavefronts exchange their partial
// results through LDS without atomics, and a pass has two barriers.  Zero words are padding: they are
// never selected, and if fewer than k words are nonzero the result is zero-padded.
struct SelectScratch {
    uint64_t sel[KB_K_MAX];
    uint32_t hist[256];
    uint32_t part[16][4];  // per wavefront: its nonzero words, AND and OR of their upper halves
    uint32_t ctl[8];       // 1 selected, 2 digit found, 3 still needed, 4 words in that bin
};

__device__ inline uint64_t shr64(uint64_t v, int s) { return s >= 64 ? 0ull : v >> s; }

// Cross-lane steps as data-parallel-primitive moves (one vector instruction each, no LDS round trip): `x` of the lane
// `shr` places down its row of 16, or lane 15 / 31 of the rows before (row_bcast), or `idle` where there is none.
template <int CTRL, int ROW_MASK> __device__ inline uint32_t dpp_or(uint32_t idle, uint32_t x)
{
    return (uint32_t)__builtin_amdgcn_update_dpp((int)idle, (int)x, CTRL, ROW_MASK, 0xf, false);
}
// Inclusive scans over the 64 lanes of a (fully active) wavefront; lane 63 ends up with the total.
__device__ inline uint32_t wave_scan_add(uint32_t x)
{
    x += dpp_or<0x111, 0xf>(0u, x);
    x += dpp_or<0x112, 0xf>(0u, x);
    x += dpp_or<0x114, 0xf>(0u, x);
    x += dpp_or<0x118, 0xf>(0u, x);
    x += dpp_or<0x142, 0xa>(0u, x);
    x += dpp_or<0x143, 0xc>(0u, x);
    return x;
}
__device__ inline uint32_t wave_scan_and(uint32_t x)
{
    x &= dpp_or<0x111, 0xf>(~0u, x);
    x &= dpp_or<0x112, 0xf>(~0u, x);
    x &= dpp_or<0x114, 0xf>(~0u, x);
    x &= dpp_or<0x118, 0xf>(~0u, x);
    x &= dpp_or<0x142, 0xa>(~0u, x);
    x &= dpp_or<0x143, 0xc>(~0u, x);
    return x;
}
__device__ inline uint32_t wave_scan_or(uint32_t x)
{
    x |= dpp_or<0x111, 0xf>(0u, x);
    x |= dpp_or<0x112, 0xf>(0u, x);
    x |= dpp_or<0x114, 0xf>(0u, x);
    x |= dpp_or<0x118, 0xf>(0u, x);
    x |= dpp_or<0x142, 0xa>(0u, x);
    x |= dpp_or<0x143, 0xc>(0u, x);
    return x;
}

// buf[0..n) in, buf[0..k) out (the rest of buf is left as it was).  All threads of the workgroup call it (at most 16
// wavefronts), converged.
__device__ inline void select_topk_desc(uint64_t *buf, int n, int k, SelectScratch *sc, int tid, int nthreads)
{
    const int lane = tid & 63, wave = tid >> 6, nwaves = nthreads >> 6;
    // ---- how many words there are, and the highest bit in which their upper halves differ ----
    {
        uint32_t cnt = 0, ahi = ~0u, ohi = 0u;
        for (int i = tid; i < n; i += nthreads) {
            const uint64_t e = buf[i];
            if (e != 0) {
                ++cnt;
                ahi &= (uint32_t)(e >> 32);
                ohi |= (uint32_t)(e >> 32);
            }
        }
        cnt = wave_scan_add(cnt);
        ahi = wave_scan_and(ahi);
        ohi = wave_scan_or(ohi);
        if (lane == 63) {
            sc->part[wave][0] = cnt;
            sc->part[wave][1] = ahi;
            sc->part[wave][2] = ohi;
        }
        for (int i = tid; i < 256; i += nthreads) sc->hist[i] = 0u;
        if (tid == 0) sc->ctl[1] = 0u;
    }
    __syncthreads();
    uint32_t nz, all_and, all_or;
    {
        // every wavefront adds the wavefronts' parts up for itself: lanes 0..15 take one each, lane 15 gets the totals
        const int w = lane & 15;
        const bool have = w < nwaves;
        uint32_t c = have ? sc->part[w][0] : 0u, a = have ? sc->part[w][1] : ~0u, o = have ? sc->part[w][2] : 0u;
        c += dpp_or<0x111, 0xf>(0u, c);
        c += dpp_or<0x112, 0xf>(0u, c);
        c += dpp_or<0x114, 0xf>(0u, c);
        c += dpp_or<0x118, 0xf>(0u, c);
        a &= dpp_or<0x111, 0xf>(~0u, a);
        a &= dpp_or<0x112, 0xf>(~0u, a);
        a &= dpp_or<0x114, 0xf>(~0u, a);
        a &= dpp_or<0x118, 0xf>(~0u, a);
        o |= dpp_or<0x111, 0xf>(0u, o);
        o |= dpp_or<0x112, 0xf>(0u, o);
        o |= dpp_or<0x114, 0xf>(0u, o);
        o |= dpp_or<0x118, 0xf>(0u, o);
        nz = (uint32_t)__builtin_amdgcn_readlane((int)c, 15);
        all_and = (uint32_t)__builtin_amdgcn_readlane((int)a, 15);
        all_or = (uint32_t)__builtin_amdgcn_readlane((int)o, 15);
    }
    // selected words: nonzero and (word >> shift) >= pref
    int shift = 0;
    uint64_t pref = 1;
    if ((int)nz > k) {
        const uint32_t diff = all_and ^ all_or;              // (the lower halves, row numbers, differ anyway)
        int hi = diff ? 64 - __builtin_clz(diff) : 32;       // bits [hi, 64) are decided and equal pref
        pref = hi >= 64 ? 0ull : (uint64_t)(all_or >> (hi - 32));
        uint32_t need = (uint32_t)k;
        for (int pass = 0; pass < 9 && hi > 0; ++pass) {
            const int width = hi < 8 ? hi : 8, lo = hi - width;
            for (int i = tid; i < n; i += nthreads) {
                const uint64_t e = buf[i];
                if (e != 0 && shr64(e, hi) == pref) atomicAdd(&sc->hist[(uint32_t)(e >> lo) & ((1u << width) - 1u)], 1u);
            }
            __syncthreads();
            if (tid < 64) {
                // lane l owns bins 4 (63 - l) .. + 3, so the scan over the lanes counts the words in higher bins; it
                // clears its bins for the next pass
                const int base = 4 * (63 - lane);
                const uint32_t c0 = sc->hist[base], c1 = sc->hist[base + 1], c2 = sc->hist[base + 2], c3 = sc->hist[base + 3];
                sc->hist[base] = 0u;
                sc->hist[base + 1] = 0u;
                sc->hist[base + 2] = 0u;
                sc->hist[base + 3] = 0u;
                const uint32_t mine = c0 + c1 + c2 + c3;
                const uint32_t incl = wave_scan_add(mine);
                uint32_t above = incl - mine;
                if (incl >= need && above < need) {
                    const uint32_t c[4] = {c0, c1, c2, c3};
                    int bin = 0;
                    uint32_t in_bin = 0;
#pragma unroll
                    for (int j = 3; j >= 0; --j) {
                        if (in_bin == 0 && above + c[j] >= need) {
                            bin = base + j;
                            in_bin = c[j];
                        } else if (in_bin == 0) {
                            above += c[j];
                        }
                    }
                    sc->ctl[2] = (uint32_t)bin;
                    sc->ctl[3] = need - above;
                    sc->ctl[4] = in_bin;
                }
            }
            __syncthreads();
            pref = (width < 64 ? pref << width : 0ull) | sc->ctl[2];
            need = sc->ctl[3];
            hi = lo;
            if (sc->ctl[4] == need) break;       // the whole bin belongs to the result
        }
        shift = hi;
    }
    for (int i = tid; i < n; i += nthreads) {
        const uint64_t e = buf[i];
        if (e != 0 && shr64(e, shift) >= pref) {
            const uint32_t slot = atomicAdd(&sc->ctl[1], 1u);
            if (slot < (uint32_t)KB_K_MAX) sc->sel[slot] = e;
        }
    }
    __syncthreads();
    const int m = (int)sc->ctl[1] < k ? (int)sc->ctl[1] : k;
    for (int t = tid; t < k; t += nthreads) {
        if (t < m) {
            const uint64_t e = sc->sel[t];
            int rank = 0;
#pragma unroll 8
            for (int j = 0; j < m; ++j) rank += sc->sel[j] > e;
            buf[rank] = e;
        } else {
            buf[t] = 0ull;
        }
    }
    __syncthreads();
}

// k-th best group maximum of the sampling pass = a lower bound of the k-th best score (k distinct
// entries reach it).  Also derives the conservative pre-filter on dot * inv_k used by the main pass:
// whenever fp32((dot*inv_k) * inv_q) >= s_thr holds, dot*inv_k >= thrp holds (2^-20 relative slack
// covers the three fp32 roundings involved).
//
// Two modes.  KEYS (weighted random selection; prep_kernel has run): the samples are candidate words of keys and the
// k-th best word is the threshold as it is.  Otherwise the kernel also does what prep_kernel does (the query's
// 1/|q|, its counters, flag and padded mask word; one workgroup per PADDED query), so that a plain query has one
// launch less, and the samples are words of s1 = dot * inv_k, which the sampling pass can form without 1/|q|.  The final
// score f(s1) = fp32(s1 * inv_q) + 0 never falls as s1 grows, so the k sampled entries with the largest words all
// have a score >= S = f(s1 of the k-th); those of them whose score equals S have an index <= the largest such
// index, and the threshold word is (S, that index): k distinct entries reach it.
struct ThresholdArgs {
    const uint64_t *samp;       // see sample_slot_index
    const void *queries;
    const uint64_t *qmask;      // or nullptr
    float *invq, *thrp;
    uint64_t *thr64, *qmask_pad, *stats;
    uint32_t *cnt, *flag, *fb_done;
    uint64_t sample_keys;
    int32_t slots, group_shift, k, Q, qpad, d, grid;
};

template <int QT, bool KEYS> __global__ __launch_bounds__(1024) void threshold_kernel(ThresholdArgs a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    uint64_t *buf = reinterpret_cast<uint64_t *>(smem_raw);
    const int q = blockIdx.x, tid = threadIdx.x, slots = a.slots, k = a.k;
    SelectScratch *sc = reinterpret_cast<SelectScratch *>(smem_raw + sizeof(uint64_t) * (slots > k ? slots : k));
    __shared__ float sh_iq;
    __shared__ uint32_t sh_low;
    // Everything the kernel reads from global memory is asked for before anything waits: the query's mask word, the
    // first two samples of every thread and (first wavefront) the query row are one memory round trip, not three.
    const int bd = (int)blockDim.x;
    uint64_t mask_word = 0ull, first0 = 0ull, first1 = 0ull;
    if (!KEYS && tid == 0 && a.qmask && q < a.Q) mask_word = a.qmask[q];
    if (KEYS || q < a.Q) {
        if (tid < slots) first0 = a.samp[sample_slot_index(tid, a.group_shift, a.qpad, q)];
        if (tid + bd < slots) first1 = a.samp[sample_slot_index(tid + bd, a.group_shift, a.qpad, q)];
    }
    if constexpr (!KEYS) {
        if (tid < CAND_SEGMENTS) a.cnt[q * CAND_SEGMENTS + tid] = 0;
        if (tid == 0) {
            a.flag[q] = 0;
            a.fb_done[q] = 0;
            a.qmask_pad[q] = mask_word;
            sh_low = 0xffffffffu;
        }
        if (q == 0 && tid < STAT_WORDS + STAT_PARTIALS) a.stats[tid] = tid == 2 ? a.sample_keys : tid == 3 ? (uint64_t)a.grid : 0ull;
        if (q >= a.Q) {         // a padding query can never pass the filter of the scan
            if (tid == 0) {
                a.invq[q] = 0.f;
                a.thr64[q] = ~0ull;
                a.thrp[q] = __builtin_inff();
            }
            return;
        }
        if (tid < 64) {
            const float inv = row_inv_norm<QT>(a.queries, q, a.d * (QT == KB_F32 ? 4 : QT == KB_BF16 ? 2 : 1), tid);
            if (tid == 0) {
                a.invq[q] = inv;
                sh_iq = inv;
            }
        }
    }
    if (tid < slots) buf[tid] = first0;
    if (tid + bd < slots) buf[tid + bd] = first1;
    for (int i = tid + 2 * bd; i < slots; i += bd) buf[i] = a.samp[sample_slot_index(i, a.group_shift, a.qpad, q)];
    __syncthreads();
    select_topk_desc(buf, slots, k, sc, tid, bd);
    uint64_t t = k <= slots ? buf[k - 1] : 0ull;
    const float iq = KEYS ? a.invq[q] : sh_iq;
    if constexpr (!KEYS) {
        if (t != 0) {
            const float s = candidate_score(t) * iq + 0.0f;
            if (tid < k && candidate_score(buf[tid]) * iq + 0.0f == s) atomicMin(&sh_low, (uint32_t)buf[tid]);
            __syncthreads();
            t = ((uint64_t)score_to_ordered(s) << 32) | sh_low;
        }
    }
    if (tid == 0) {
        float tp = -__builtin_inff();
        if (KEYS) {
            // keys are compared as they are: a word at or above t has a key at or above t's key
            if (t != 0) tp = candidate_score(t);
        } else if (t != 0 && iq > 0.f) {
            const float x = candidate_score(t) / iq;
            tp = x - fabsf(x) * 0x1p-20f - 1e-30f;
        }
        a.thr64[q] = t;
        a.thrp[q] = tp;
    }
}

// ------------------------------------------------------------------------------------------------
// finalize: select each query's best k in order; a query whose list overflowed is resolved by an
// exhaustive scan of all keys (shared by fb_parts workgroups) that uses the same MFMA sequence per output
// element as the scan kernel, so both paths produce bit-identical scores.
// ------------------------------------------------------------------------------------------------
struct FinalArgs {
    const void *keys;
    const float *inv_norm;
    const uint64_t *tags;
    const void *queries;
    const uint64_t *qmask;
    const float *invq;
    const uint64_t *cand;
    const uint32_t *cnt;
    const uint32_t *flag;
    uint64_t *stats;
    int32_t *out_index;
    float *out_score;
    int64_t n_keys;
    int32_t d, k, cand_cap;
    DrawArgs draw;
    uint32_t *fb_done;        // [Q] arrivals of the parts of an exhaustive scan (zero before the launch)
    uint64_t *fb_lists;       // [Q][fb_parts][k] their partial results
    int32_t fb_parts;
    const uint64_t *thr64;    // [Q] threshold words of the scan
    int32_t raw;              // the lists hold dot * inv_k products (plain queries), not finished candidate words
};

// KT = KT_FP8_Q8 stands for fp8 keys with fp8 queries (one fp8 matrix instruction per 64-byte chunk, as in the scan).
constexpr int KT_FP8_Q8 = 3;
typedef int i32x8 __attribute__((ext_vector_type(8)));
template <int KT> __device__ void exhaustive_query(const FinalArgs &a, int q, uint64_t *buf, uint32_t *ctl, SelectScratch *sc, int64_t row_begin,
                                                   int64_t row_end, const float *inv_q = nullptr)
{
    constexpr bool Q8 = KT == KT_FP8_Q8;
    constexpr int KTT = Q8 ? (int)KB_FP8_E4M3 : KT;
    constexpr int KEY_BYTES = KeyTraits<KTT>::KEY_BYTES, QRY_BYTES = Q8 ? 1 : KeyTraits<KTT>::QRY_BYTES, BMUL = QRY_BYTES / KEY_BYTES;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, lrow = lane & 31, half = lane >> 5;
    const int cap = a.cand_cap;
    const bool filter = a.qmask != nullptr;
    const uint64_t qm = filter ? a.qmask[q] : 0;
    const float iq = inv_q ? *inv_q : a.invq[q];
    const size_t key_row_bytes = (size_t)a.d * KEY_BYTES;
    const unsigned char *qrow = static_cast<const unsigned char *>(a.queries) + (size_t)q * a.d * QRY_BYTES;
    const int n_groups = (int)(key_row_bytes / (Q8 ? 64 : 32));
    uint64_t *thr_local = reinterpret_cast<uint64_t *>(ctl + 2);   // ctl[0] = count, ctl[2..3] = threshold word
    if (tid == 0) {
        ctl[0] = 0;
        *thr_local = 0;
    }
    __syncthreads();
    for (int64_t row0 = row_begin; row0 < row_end; row0 += 128) {
        int64_t my_row = row0 + wave * 32 + lrow;
        if (my_row >= row_end) my_row = row_end - 1;
        const unsigned char *krow = static_cast<const unsigned char *>(a.keys) + (size_t)my_row * key_row_bytes + half * 16;
        f32x16 acc;
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[i] = 0.f;
        // The loads of UNR groups go out before their matrix instructions (the order of the accumulation does not
        // change): one memory round trip per UNR groups instead of one per group (16 where a group is two registers
        // quadruples, 8 where it is three or four).
        constexpr int UNR = (Q8 || BMUL == 2) ? 8 : 16;
        if constexpr (Q8) {
            // one fp8 matrix instruction per 64-byte chunk: lane half h supplies bytes [32h, 32h+32) of its key row
            // and of the query row, the operand layout the scan uses, so both paths give the same bits
            const unsigned char *kp = krow + half * 16;
            auto step = [&](const u32x4 &a0, const u32x4 &a1, const u32x4 &b0, const u32x4 &b1) {
                const i32x8 av = {(int)a0[0], (int)a0[1], (int)a0[2], (int)a0[3], (int)a1[0], (int)a1[1], (int)a1[2], (int)a1[3]};
                const i32x8 bv = {(int)b0[0], (int)b0[1], (int)b0[2], (int)b0[3], (int)b1[0], (int)b1[1], (int)b1[2], (int)b1[3]};
                acc = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(av, bv, acc, 0, 0, 0, 0, 0, 0);
            };
            int g = 0;
            for (; g + UNR <= n_groups; g += UNR) {
                u32x4 a0[UNR], a1[UNR], b0[UNR], b1[UNR];
#pragma unroll
                for (int u = 0; u < UNR; ++u) {
                    a0[u] = *reinterpret_cast<const u32x4 *>(kp + (size_t)(g + u) * 64);
                    a1[u] = *reinterpret_cast<const u32x4 *>(kp + (size_t)(g + u) * 64 + 16);
                    b0[u] = *reinterpret_cast<const u32x4 *>(qrow + (size_t)(g + u) * 64 + half * 32);
                    b1[u] = *reinterpret_cast<const u32x4 *>(qrow + (size_t)(g + u) * 64 + half * 32 + 16);
                }
#pragma unroll
                for (int u = 0; u < UNR; ++u) step(a0[u], a1[u], b0[u], b1[u]);
            }
            for (; g < n_groups; ++g)
                step(*reinterpret_cast<const u32x4 *>(kp + (size_t)g * 64), *reinterpret_cast<const u32x4 *>(kp + (size_t)g * 64 + 16),
                     *reinterpret_cast<const u32x4 *>(qrow + (size_t)g * 64 + half * 32), *reinterpret_cast<const u32x4 *>(qrow + (size_t)g * 64 + half * 32 + 16));
        } else {
            const unsigned char *qbase = qrow + half * 16 * BMUL;
            int g = 0;
            for (; g + UNR <= n_groups; g += UNR) {
                u32x4 av[UNR], b0[UNR], b1[UNR];
#pragma unroll
                for (int u = 0; u < UNR; ++u) {
                    av[u] = *reinterpret_cast<const u32x4 *>(krow + (size_t)(g + u) * 32);
                    const unsigned char *qp = qbase + (size_t)(g + u) * 32 * BMUL;
                    b0[u] = *reinterpret_cast<const u32x4 *>(qp);
                    b1[u] = BMUL == 2 ? *reinterpret_cast<const u32x4 *>(qp + 16) : b0[u];
                }
#pragma unroll
                for (int u = 0; u < UNR; ++u) Mma<KTT>::run(acc, Mma<KTT>::prepare(av[u]), b0[u], b1[u]);
            }
            for (; g < n_groups; ++g) {
                const u32x4 av = *reinterpret_cast<const u32x4 *>(krow + (size_t)g * 32);
                const unsigned char *qp = qbase + (size_t)g * 32 * BMUL;
                const u32x4 b0 = *reinterpret_cast<const u32x4 *>(qp);
                const u32x4 b1 = BMUL == 2 ? *reinterpret_cast<const u32x4 *>(qp + 16) : b0;
                Mma<KTT>::run(acc, Mma<KTT>::prepare(av), b0, b1);
            }
        }
        // every column holds the same query; lanes 0..15 of each half own one row each
        float v = acc[0];
#pragma unroll
        for (int i = 1; i < 16; ++i) v = (lrow == i) ? acc[i] : v;
        if (lrow < 16) {
            const int64_t row = row0 + wave * 32 + 8 * (lrow >> 2) + 4 * half + (lrow & 3);
            if (row < row_end && !row_removed(a.inv_norm[row]) && (!filter || (a.tags[row] & qm) != 0)) {
                float value = final_score(v, a.inv_norm[row], iq);
                if (a.draw.enabled) value = draw_key_of(value, a.draw, a.draw.first_query + (uint32_t)q, row);
                const uint64_t cw = pack_candidate(value, (uint32_t)row);
                if (cw > *thr_local && value > -__builtin_inff()) {
                    const uint32_t pos = atomicAdd(&ctl[0], 1u);
                    buf[pos] = cw;      // pos < cap: at most 128 appends between compactions
                }
            }
        }
        __syncthreads();
        const uint32_t n = ctl[0];
        if (n + 128 > (uint32_t)cap) {      // uniform: compact to the best k (sorted into buf[0..k))
            select_topk_desc(buf, (int)n, a.k, sc, tid, 256);
            if (tid == 0) {
                ctl[0] = n < (uint32_t)a.k ? n : (uint32_t)a.k;
                *thr_local = n >= (uint32_t)a.k ? buf[a.k - 1] : 0ull;
            }
            __syncthreads();
        }
    }
    select_topk_desc(buf, (int)ctl[0], a.k, sc, tid, 256);      // buf[0..k): the result in order, zero words where there is none
}

template <int KT> __global__ __launch_bounds__(256) void finalize_kernel(FinalArgs a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    uint64_t *buf = reinterpret_cast<uint64_t *>(smem_raw);
    uint32_t *ctl = reinterpret_cast<uint32_t *>(smem_raw + sizeof(uint64_t) * a.cand_cap);
    SelectScratch *sc = reinterpret_cast<SelectScratch *>(smem_raw + sizeof(uint64_t) * a.cand_cap + 16);
    const int q = blockIdx.x, part = blockIdx.y, tid = threadIdx.x;
    // (the segment counters are asked for together with the flag: one memory round trip instead of two on the path
    // of every query; the parts that turn out to have nothing to do have read 64 bytes in vain)
    uint32_t seg_cnt[CAND_SEGMENTS];
    {
        const u32x4 *cp = reinterpret_cast<const u32x4 *>(a.cnt + (size_t)q * CAND_SEGMENTS);
#pragma unroll
        for (int v = 0; v < CAND_SEGMENTS / 4; ++v) {
            const u32x4 c4 = cp[v];
            seg_cnt[4 * v] = c4[0];
            seg_cnt[4 * v + 1] = c4[1];
            seg_cnt[4 * v + 2] = c4[2];
            seg_cnt[4 * v + 3] = c4[3];
        }
    }
    const bool flagged = a.flag[q] != 0 && a.n_keys > 0;
    if (!flagged && part != 0) return;
    if (flagged) {
        // The grid has fb_parts workgroups per query; for a flagged query each scans its share of the rows and leaves
        // its best k as a sorted list, and the one that arrives last merges the lists.  (One workgroup alone would
        // read the whole knowledge base at the speed of a single compute unit.)
        const int64_t len = ((a.n_keys + a.fb_parts - 1) / a.fb_parts + 127) / 128 * 128;
        const int64_t begin = (int64_t)part * len, end = begin + len < a.n_keys ? begin + len : a.n_keys;
        uint64_t *mine = a.fb_lists + ((size_t)q * a.fb_parts + part) * a.k;
        if (begin < end) exhaustive_query<KT>(a, q, buf, ctl, sc, begin, end);
        if (tid < a.k) mine[tid] = begin < end ? buf[tid] : 0ull;
        __threadfence();                // the list is visible device-wide before the arrival is counted
        __syncthreads();
        if (tid == 0) ctl[1] = atomicAdd(&a.fb_done[q], 1u);
        __syncthreads();
        if (ctl[1] != (uint32_t)a.fb_parts - 1) return;
        __threadfence();
        const int n = a.fb_parts * a.k;                                  // <= cand_cap words
        const uint64_t *lists = a.fb_lists + (size_t)q * a.fb_parts * a.k;
        for (int i = tid; i < n; i += 256) buf[i] = __builtin_nontemporal_load(lists + i);
        __syncthreads();
        select_topk_desc(buf, n, a.k, sc, tid, 256);
        if (tid == 0) atomicAdd(reinterpret_cast<unsigned long long *>(a.stats + 1), 1ull);
    } else {
        // gather the query's segments into one contiguous list
        const uint32_t seg_cap = (uint32_t)a.cand_cap / CAND_SEGMENTS;
        uint32_t seg_n[CAND_SEGMENTS], seg_off[CAND_SEGMENTS], n = 0;
#pragma unroll
        for (int sg = 0; sg < CAND_SEGMENTS; ++sg) {
            uint32_t c = a.n_keys > 0 ? seg_cnt[sg] : 0;
            seg_n[sg] = c < seg_cap ? c : seg_cap;
            seg_off[sg] = n;
            n += seg_n[sg];
        }
        // Thread t takes positions t, t + 256, ... of the gathered list, four at a time: their loads are in flight
        // together, where a loop over the segments would wait for one segment's words before asking for the next.
        // A plain scan leaves (dot * inv_k, row) of live rows: each candidate is finished here as the scan's exact test
        // would have: the final score from the same three fp32 operations every kernel uses, nothing below the
        // threshold word.  What fails becomes a zero word, which sorts last.
        const float iq = a.invq[q];
        const uint64_t t64 = a.raw ? a.thr64[q] : 0ull;
        const uint64_t *lists = a.cand + (size_t)q * a.cand_cap;
        for (uint32_t j0 = tid; j0 < n; j0 += 4 * 256) {
            uint64_t w[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const uint32_t j = j0 + u * 256;
                uint32_t sg = 0, off = 0;
#pragma unroll
                for (int s2 = 1; s2 < CAND_SEGMENTS; ++s2) {
                    const bool past = j >= seg_off[s2];
                    sg += past ? 1u : 0u;
                    off = past ? seg_off[s2] : off;
                }
                w[u] = j < n ? lists[sg * seg_cap + (j - off)] : 0ull;
            }
            if (a.raw) {
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const uint64_t c = pack_candidate(raw_candidate_product(w[u]) * iq + 0.0f, candidate_index(w[u]));
                    w[u] = (w[u] != 0ull && c >= t64) ? c : 0ull;
                }
            }
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (j0 + u * 256 < n) buf[j0 + u * 256] = w[u];
        }
        __syncthreads();
        select_topk_desc(buf, (int)n, a.k, sc, tid, 256);
    }
    if (tid < a.k) {
        const uint64_t cw = tid < a.cand_cap ? buf[tid] : 0ull;
        a.out_index[(size_t)q * a.k + tid] = cw ? (int32_t)candidate_index(cw) : -1;
        a.out_score[(size_t)q * a.k + tid] = cw ? candidate_score(cw) : -__builtin_inff();
    }
}

// ------------------------------------------------------------------------------------------------
// Two-stage retrieval, second stage: exact top-k of one query over the rows of the clusters it probes.
// ------------------------------------------------------------------------------------------------
constexpr int PROBE_CAP = 1024;        // LDS candidate buffer of a partial scan (words); k <= 128 fits eight times
constexpr int PROBE_MAX_LISTS = 64;    // partial lists per query that the merge can take: 64 x 128 = MAX_CAND_CAP words

// Block (p, s, q): part s of `splits` of the rows of cluster probe[q][p], scored exactly as the scan kernels score
// (same MFMA sequence per element), best k written as a sorted list of candidate words (zero = no entry).
// Without cluster_offsets the one "cluster" is the whole knowledge base (the path of small knowledge bases).
// Every block computes 1/|q| of its query itself (one wavefront, the row-norm routine every path uses: the same bits),
// which saves the launch that would do it once per query: these calls are bound by the latency of their launches.
// stats (optional): the diagnostics of a query that took this path: no candidates, no sampling, one workgroup per block.
template <int KT> __global__ __launch_bounds__(256) void probe_scan_kernel(FinalArgs a, const int64_t *cluster_offsets, int n_clusters,
                                                                         const int32_t *probe, int nprobe, int splits, uint64_t *lists, uint64_t *stats)
{
    constexpr int QT = KT == KB_F32 ? (int)KB_F32 : KT == KT_FP8_Q8 ? (int)KB_FP8_E4M3 : (int)KB_BF16;     // type of the queries
    __shared__ __attribute__((aligned(16))) uint64_t buf[PROBE_CAP];
    __shared__ uint32_t ctl[4];
    __shared__ SelectScratch sc;
    __shared__ float inv_q;
    const int p = blockIdx.x, s = blockIdx.y, q = blockIdx.z, tid = threadIdx.x;
    if (stats && p == 0 && s == 0 && q == 0 && tid < STAT_WORDS + STAT_PARTIALS)
        stats[tid] = tid == 3 ? (uint64_t)gridDim.x * gridDim.y * gridDim.z : 0ull;
    uint64_t *out = lists + ((size_t)q * nprobe * splits + (size_t)p * splits + s) * a.k;
    const int c = cluster_offsets ? probe[(size_t)q * nprobe + p] : 0;
    bool first = true;          // a cluster named twice is scanned once (the merge takes distinct entries)
    for (int e = 0; cluster_offsets && e < p; ++e) first = first && probe[(size_t)q * nprobe + e] != c;
    int64_t begin = 0, end = 0;
    if (first && c >= 0 && c < n_clusters) {
        const int64_t cb = cluster_offsets ? cluster_offsets[c] : 0, ce = cluster_offsets ? cluster_offsets[c + 1] : a.n_keys;
        if (cb >= 0 && ce <= a.n_keys && cb < ce) {
            const int64_t len = ((ce - cb + splits - 1) / splits + 127) / 128 * 128;    // whole steps of the scorer
            begin = cb + (int64_t)s * len;
            end = begin + len < ce ? begin + len : ce;
        }
    }
    if (begin >= end) {         // workgroup-uniform
        if (tid < a.k) out[tid] = 0ull;
        return;
    }
    if (tid < 64) {
        const float inv = row_inv_norm<QT>(a.queries, q, a.d * (QT == KB_F32 ? 4 : QT == KB_BF16 ? 2 : 1), tid);
        if (tid == 0) inv_q = inv;
    }
    __syncthreads();
    exhaustive_query<KT>(a, q, buf, ctl, &sc, begin, end, &inv_q);
    if (tid < a.k) out[tid] = buf[tid];
}

__global__ __launch_bounds__(256) void probe_merge_kernel(const uint64_t *lists, int n_lists, int k, int32_t *out_index, float *out_score)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    uint64_t *buf = reinterpret_cast<uint64_t *>(smem_raw);
    const int n = n_lists * k, q = blockIdx.x, tid = threadIdx.x;
    SelectScratch *sc = reinterpret_cast<SelectScratch *>(smem_raw + sizeof(uint64_t) * (size_t)(n > k ? n : k) + 16);
    for (int i = tid; i < n; i += 256) buf[i] = lists[(size_t)q * n + i];
    __syncthreads();
    select_topk_desc(buf, n, k, sc, tid, 256);
    if (tid < k) {
        const uint64_t cw = buf[tid];
        out_index[(size_t)q * k + tid] = cw ? (int32_t)candidate_index(cw) : -1;
        out_score[(size_t)q * k + tid] = cw ? candidate_score(cw) : -__builtin_inff();
    }
}

hipError_t launch_scan(kb_dtype_t dt, int config, int family, bool sample, int grid, const ScanArgs &a, hipStream_t s)
{
    if (family == 4)
        return dt == KB_BF16 ? launch_scan_wide_bf16(config, sample, grid, a, s)
               : dt == KB_FP8_E4M3 ? launch_scan_wide_fp8(config, sample, grid, a, s) : hipErrorInvalidValue;
    if (family == 3)
        return dt == KB_BF16 ? launch_scan_sp_bf16(config, sample, grid, a, s)
               : dt == KB_FP8_E4M3 ? launch_scan_sp_fp8(config, sample, grid, a, s) : hipErrorInvalidValue;
    switch (dt) {
    case KB_F32: return launch_scan_f32(config, sample, grid, a, s);
    case KB_BF16: return launch_scan_bf16(config, sample, grid, a, s);
    default: return launch_scan_fp8(config, sample, grid, a, s);
    }
}

bool valid_dtype(int t) { return t == KB_F32 || t == KB_BF16 || t == KB_FP8_E4M3; }

}  // namespace

// ------------------------------------------------------------------------------------------------
// C ABI
// ------------------------------------------------------------------------------------------------
extern "C" {

kb_status_t kb_create(kb_t **out, int32_t d, kb_dtype_t key_dtype, int64_t capacity, void *keys_dev, float *row_scale_dev,
                      float *inv_norm_dev, uint64_t *tags_dev)
{
    if (!out) return KB_ERR_NULL;
    *out = nullptr;
    if (!valid_dtype((int)key_dtype)) return KB_ERR_DTYPE;
    if (!keys_dev || !inv_norm_dev) return KB_ERR_NULL;
    if (key_dtype == KB_FP8_E4M3 && !row_scale_dev) return KB_ERR_NULL;
    if (key_dtype != KB_FP8_E4M3 && row_scale_dev) return KB_ERR_INVALID_ARG;
    const int granule = key_dtype == KB_F32 ? 32 : 64;
    if (d <= 0 || d % granule != 0 || d > 16384) return KB_ERR_INVALID_ARG;
    if (capacity < 1 || capacity >= ((int64_t)1 << 31)) return KB_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(keys_dev) & 15) != 0) return KB_ERR_INVALID_ARG;
    kb *h = new (std::nothrow) kb();
    if (!h) return KB_ERR_INVALID_ARG;
    h->d = d;
    h->dtype = key_dtype;
    h->capacity = capacity;
    h->n = h->n_normalized = 0;
    h->keys = keys_dev;
    h->row_scale = row_scale_dev;
    h->inv_norm = inv_norm_dev;
    h->tags = tags_dev;
    h->tune_sample_keys = h->tune_config = h->tune_wg_per_cu = h->tune_no_small_path = 0;
    h->prof_events = nullptr;
    h->prof_max = h->prof_used = 0;
    h->prof_stride = 1;
    h->prof_seen = 0;
    *out = h;
    return KB_OK;
}

kb_status_t kb_append(kb_t *kb, const void *rows_dev, const float *row_scale_dev, const uint64_t *tags_dev, int64_t n,
                      void *hip_stream, int64_t *first_index_out)
{
    if (!kb) return KB_ERR_NULL;
    if (n < 0) return KB_ERR_INVALID_ARG;
    if (n == 0) {
        if (first_index_out) *first_index_out = kb->n;
        return KB_OK;
    }
    if (!rows_dev) return KB_ERR_NULL;
    if (kb->dtype == KB_FP8_E4M3 && !row_scale_dev) return KB_ERR_NULL;
    if (kb->tags && !tags_dev) return KB_ERR_NULL;
    if (kb->n + n > kb->capacity) return KB_ERR_CAPACITY;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const size_t row_bytes = (size_t)kb->d * key_bytes(kb->dtype);
    void *dst = static_cast<unsigned char *>(kb->keys) + (size_t)kb->n * row_bytes;
    if (dst != rows_dev && hipMemcpyAsync(dst, rows_dev, row_bytes * n, hipMemcpyDeviceToDevice, s) != hipSuccess)
        return KB_ERR_DEVICE;
    if (kb->dtype == KB_FP8_E4M3 && kb->row_scale + kb->n != row_scale_dev &&
        hipMemcpyAsync(kb->row_scale + kb->n, row_scale_dev, sizeof(float) * n, hipMemcpyDeviceToDevice, s) != hipSuccess)
        return KB_ERR_DEVICE;
    if (kb->tags && kb->tags + kb->n != tags_dev &&
        hipMemcpyAsync(kb->tags + kb->n, tags_dev, sizeof(uint64_t) * n, hipMemcpyDeviceToDevice, s) != hipSuccess)
        return KB_ERR_DEVICE;
    if (first_index_out) *first_index_out = kb->n;
    kb->n += n;
    return KB_OK;
}

kb_status_t kb_normalize(kb_t *kb, void *hip_stream)
{
    if (!kb) return KB_ERR_NULL;
    const int64_t begin = kb->n_normalized, end = kb->n;
    if (end <= begin) return KB_OK;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const unsigned grid = (unsigned)ceil_div(end - begin, 4);
    switch (kb->dtype) {
    case KB_F32: hipLaunchKernelGGL(row_norm_kernel<KB_F32>, dim3(grid), dim3(256), 0, s, kb->keys, begin, end, kb->d, kb->inv_norm); break;
    case KB_BF16: hipLaunchKernelGGL(row_norm_kernel<KB_BF16>, dim3(grid), dim3(256), 0, s, kb->keys, begin, end, kb->d, kb->inv_norm); break;
    default: hipLaunchKernelGGL(row_norm_kernel<KB_FP8_E4M3>, dim3(grid), dim3(256), 0, s, kb->keys, begin, end, kb->d, kb->inv_norm); break;
    }
    if (hipGetLastError() != hipSuccess) return KB_ERR_DEVICE;
    kb->n_normalized = end;
    return KB_OK;
}

// ------------------------------------------------------------------------------------------------
// Two-stage retrieval, second stage (host side)
// ------------------------------------------------------------------------------------------------
namespace {

// Parts a cluster's rows are split into, so that a small batch still fills the device: a function of (Q, nprobe) only.
int probe_splits(int Q, int nprobe)
{
    int64_t s = (4 * (int64_t)DEVICE_CUS + (int64_t)Q * nprobe - 1) / ((int64_t)Q * nprobe);
    if (s > 16) s = 16;
    if (s > PROBE_MAX_LISTS / nprobe) s = PROBE_MAX_LISTS / nprobe;
    return s < 1 ? 1 : (int)s;
}

struct ProbePlan {
    int splits;
    size_t off_invq, off_lists, total;
};

bool make_probe_plan(int32_t Q, int32_t k, int32_t nprobe, ProbePlan *out)
{
    if (Q < 1 || Q > 65535 || k < 1 || k > KB_K_MAX || nprobe < 1 || nprobe > PROBE_MAX_LISTS) return false;
    ProbePlan p;
    p.splits = probe_splits(Q, nprobe);
    p.off_invq = 0;
    p.off_lists = align_up((size_t)Q * 4);
    p.total = p.off_lists + align_up((size_t)Q * nprobe * p.splits * k * 8);
    *out = p;
    return true;
}


// The two launches behind kb_query_probe; also the whole pipeline of kb_query on a small knowledge base
// (cluster_offsets == nullptr: one "cluster" = every row, nprobe = 1, `stats` zeroed for kb_query_counters).
kb_status_t launch_probe(kb *h, bool timed_scan, const void *queries_dev, kb_dtype_t q_dtype, bool q8, int32_t Q, const uint64_t *qmask_dev, int32_t k,
                         const int64_t *cluster_offsets_dev, int32_t n_clusters, const int32_t *probe_dev, int32_t nprobe, int splits, float *invq,
                         uint64_t *lists, uint64_t *stats, int32_t *indices_out_dev, float *scores_out_dev, hipStream_t s)
{
    FinalArgs f;
    memset(&f, 0, sizeof f);
    f.keys = h->keys;
    f.inv_norm = h->inv_norm;
    f.tags = h->tags;
    f.queries = queries_dev;
    f.qmask = qmask_dev;
    f.invq = invq;
    f.n_keys = h->n;
    f.d = h->d;
    f.k = k;
    f.cand_cap = PROBE_CAP;
    const dim3 grid(nprobe, splits, Q);
    const bool timed = timed_scan && h->prof_events && h->prof_used < h->prof_max && h->prof_seen++ % h->prof_stride == h->prof_stride / 2;     // the scoring kernel stands for the scan
    if (timed && hipEventRecord(h->prof_events[2 * h->prof_used], s) != hipSuccess) return KB_ERR_DEVICE;
    switch (q8 ? KT_FP8_Q8 : (int)h->dtype) {
    case KB_F32: hipLaunchKernelGGL(probe_scan_kernel<KB_F32>, grid, dim3(256), 0, s, f, cluster_offsets_dev, n_clusters, probe_dev, nprobe, splits, lists, stats); break;
    case KB_BF16: hipLaunchKernelGGL(probe_scan_kernel<KB_BF16>, grid, dim3(256), 0, s, f, cluster_offsets_dev, n_clusters, probe_dev, nprobe, splits, lists, stats); break;
    case KB_FP8_E4M3: hipLaunchKernelGGL(probe_scan_kernel<KB_FP8_E4M3>, grid, dim3(256), 0, s, f, cluster_offsets_dev, n_clusters, probe_dev, nprobe, splits, lists, stats); break;
    default: hipLaunchKernelGGL(probe_scan_kernel<KT_FP8_Q8>, grid, dim3(256), 0, s, f, cluster_offsets_dev, n_clusters, probe_dev, nprobe, splits, lists, stats); break;
    }
    if (timed) {
        if (hipEventRecord(h->prof_events[2 * h->prof_used + 1], s) != hipSuccess) return KB_ERR_DEVICE;
        ++h->prof_used;
    }
    const int n_lists = nprobe * splits;
    const size_t merge_lds = sizeof(uint64_t) * (size_t)(n_lists * k > k ? n_lists * k : k) + 16 + sizeof(SelectScratch);
    static LdsAllowed merge_allowed;
    if (allow_dynamic_lds(reinterpret_cast<const void *>(&probe_merge_kernel), merge_allowed, MAX_CAND_CAP * 8 + 16 + sizeof(SelectScratch)) != hipSuccess)
        return KB_ERR_DEVICE;
    hipLaunchKernelGGL(probe_merge_kernel, dim3(Q), dim3(256), merge_lds, s, lists, n_lists, k, indices_out_dev, scores_out_dev);
    return hipGetLastError() == hipSuccess ? KB_OK : KB_ERR_DEVICE;
}

// A small knowledge base is scored whole by the same two launches: parts of 128 or 256 rows (one or two steps of the scorer), no
// sampling pass, no candidate lists.  Same scores, same order: results do not depend on which path ran.
constexpr int64_t SMALL_ROWS = 16384;
constexpr int SMALL_BLOCKS = 1024;
int small_path_parts(const kb *h, int64_t n, int32_t Q, bool draw)
{
    if (draw || h->tune_no_small_path || h->tune_config || h->tune_sample_keys || h->tune_wg_per_cu) return 0;
    if (n < 1 || n > SMALL_ROWS || Q > 65535) return 0;
    int64_t parts = (n + 127) / 128;       // one step of the scorer per part up to 8192 rows, two beyond
    if (parts > PROBE_MAX_LISTS) parts = PROBE_MAX_LISTS;
    return parts * Q <= SMALL_BLOCKS ? (int)parts : 0;
}

struct SmallPlan {
    size_t off_invq, off_lists, total;
};
SmallPlan make_small_plan(int32_t Q, int32_t k, int parts)
{
    SmallPlan p;
    p.off_invq = align_up(sizeof(uint64_t) * (STAT_WORDS + STAT_PARTIALS));      // the diagnostics come first, as always
    p.off_lists = p.off_invq + align_up((size_t)Q * 4);
    p.total = p.off_lists + align_up((size_t)Q * parts * k * 8);
    return p;
}

}  // namespace

size_t kb_query_workspace_bytes(const kb_t *kb, int32_t Q, int32_t k)
{
    if (!kb || Q < 1 || k < 1 || k > KB_K_MAX) return 0;
    // Every combination of kernels a query on this handle can run (the choice depends on the row count only through
    // the two sides of WIDE128_MIN_ROWS, and on the kind of query), each bounded over all row counts.
    Sizes m;
    memset(&m, 0, sizeof m);
    bool any = false;
    const int64_t ns[2] = {1, kb->capacity};
    for (int64_t n : ns)
        for (int kind = 0; kind < 4; ++kind) {      // plain, weighted random selection, fp8 queries, both
            Choice c;
            if (!choose_kernels(kb, n, Q, (kind & 1) != 0, (kind & 2) != 0, &c)) continue;
            bound_sizes(kb, c, Q, k, (kind & 1) != 0, m);
            any = true;
        }
    if (!any) return 0;
    Plan p;
    lay_out(m, &p);
    const size_t small = make_small_plan(Q, k, PROBE_MAX_LISTS).total;      // the path of small knowledge bases
    return p.total > small ? p.total : small;
}

size_t kb_query_plan_bytes(const kb_t *kb, int64_t n, int32_t Q, int32_t k, int32_t kind)
{
    if (!kb || n < 0 || n > kb->capacity || Q < 1 || k < 1 || k > KB_K_MAX || kind < 0 || kind > 3) return 0;
    if (const int parts = small_path_parts(kb, n, Q, (kind & 1) != 0)) return make_small_plan(Q, k, parts).total;
    Plan p;
    return make_plan(kb, n, Q, k, (kind & 1) != 0, (kind & 2) != 0, &p) ? p.total : 0;
}

// kb_query and kb_query_sampled: the same pipeline; `gain_dev` != nullptr selects the weighted random selection.
static kb_status_t run_query(kb_t *kb, const void *queries_dev, kb_dtype_t q_dtype, int32_t Q, const uint64_t *qmask_dev, int32_t k,
                             const float *gain_dev, float temperature, uint64_t seed, int32_t first_query,
                             int32_t *indices_out_dev, float *scores_out_dev, void *workspace_dev, size_t workspace_bytes,
                             void *hip_stream)
{
    const bool draw = gain_dev != nullptr;
    if (!kb || !queries_dev || !indices_out_dev || !scores_out_dev) return KB_ERR_NULL;
    if (!valid_dtype((int)q_dtype)) return KB_ERR_DTYPE;
    const kb_dtype_t want_q = kb->dtype == KB_F32 ? KB_F32 : KB_BF16;
    const bool q8 = kb->dtype == KB_FP8_E4M3 && q_dtype == KB_FP8_E4M3;     // fp8 queries against fp8 keys
    if (q_dtype != want_q && !q8) return KB_ERR_DTYPE;
    if (Q < 1 || k < 1 || k > KB_K_MAX) return KB_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(queries_dev) & 15) != 0) return KB_ERR_INVALID_ARG;
    if (qmask_dev && !kb->tags) return KB_ERR_NO_TAGS;
    if (kb->n_normalized != kb->n) return KB_ERR_NOT_NORMALIZED;
    if (!workspace_dev || (reinterpret_cast<uintptr_t>(workspace_dev) & (WS_ALIGN - 1)) != 0) return KB_ERR_WORKSPACE;
    if (const int parts = small_path_parts(kb, kb->n, Q, draw)) {
        const SmallPlan sp = make_small_plan(Q, k, parts);
        if (workspace_bytes < sp.total) return KB_ERR_WORKSPACE;
        unsigned char *w = static_cast<unsigned char *>(workspace_dev);
        return launch_probe(kb, true, queries_dev, q_dtype, q8, Q, qmask_dev, k, nullptr, 1, nullptr, 1, parts, reinterpret_cast<float *>(w + sp.off_invq),
                            reinterpret_cast<uint64_t *>(w + sp.off_lists), reinterpret_cast<uint64_t *>(w), indices_out_dev, scores_out_dev,
                            static_cast<hipStream_t>(hip_stream));
    }
    Plan p;
    if (!make_plan(kb, kb->n, Q, k, draw, q8, &p)) return KB_ERR_INVALID_ARG;
    if (workspace_bytes < p.total) return KB_ERR_WORKSPACE;

    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    unsigned char *ws = static_cast<unsigned char *>(workspace_dev);
    float *invq = reinterpret_cast<float *>(ws + p.off_invq);
    uint64_t *thr64 = reinterpret_cast<uint64_t *>(ws + p.off_thr64);
    float *thrp = reinterpret_cast<float *>(ws + p.off_thrp);
    uint32_t *cnt = reinterpret_cast<uint32_t *>(ws + p.off_cnt);
    uint32_t *flag = reinterpret_cast<uint32_t *>(ws + p.off_flag);
    uint32_t *fb_done = reinterpret_cast<uint32_t *>(ws + p.off_fb_done);
    uint64_t *stats = reinterpret_cast<uint64_t *>(ws + p.off_stats);
    uint64_t *qmask_pad = reinterpret_cast<uint64_t *>(ws + p.off_qmask);
    uint64_t *samp = reinterpret_cast<uint64_t *>(ws + p.off_samp);
    Record *regions = reinterpret_cast<Record *>(ws + p.off_regions);
    uint64_t *cand = reinterpret_cast<uint64_t *>(ws + p.off_cand);
    float *log_gain = reinterpret_cast<float *>(ws + p.off_lgain);

    DrawArgs dr;
    memset(&dr, 0, sizeof dr);
    if (draw) {
        dr.log_gain = log_gain;
        dr.inv_t = 1.0f / temperature;
        dr.seed_lo = (uint32_t)seed;
        dr.seed_hi = (uint32_t)(seed >> 32);
        dr.first_query = (uint32_t)first_query;
        dr.enabled = 1;
        const int64_t n_padded = ceil_div(kb->n > 0 ? kb->n : 1, 256) * 256 + 256;
        hipLaunchKernelGGL(log_gain_kernel, dim3((unsigned)ceil_div(n_padded, 256)), dim3(256), 0, s, gain_dev, kb->n, n_padded, log_gain);
        if (hipGetLastError() != hipSuccess) return KB_ERR_DEVICE;
    }

    // Query norms and per-call counters: the threshold kernel sets them when there is a sampling pass on scores;
    // otherwise (no sampling pass, or the weighted random selection, whose sampling pass needs 1/|q|) this launch does.
    const bool sampled = kb->n > 0 && p.sample_tiles > 0;
    if (!sampled || draw) {
        const int n_init = p.qpad > STAT_WORDS + STAT_PARTIALS ? p.qpad : STAT_WORDS + STAT_PARTIALS;
        const int blocks_rows = (int)ceil_div(p.qpad, 4), blocks_init = (int)ceil_div(n_init, 256);
        const unsigned grid = blocks_rows > blocks_init ? blocks_rows : blocks_init;
        if (q_dtype == KB_F32)
            hipLaunchKernelGGL(prep_kernel<KB_F32>, dim3(grid), dim3(256), 0, s, queries_dev, Q, p.qpad, kb->d, invq, thr64, thrp, cnt, flag, stats, (uint64_t)p.sample_keys, qmask_dev, qmask_pad, p.grid, fb_done);
        else if (q_dtype == KB_FP8_E4M3)
            hipLaunchKernelGGL(prep_kernel<KB_FP8_E4M3>, dim3(grid), dim3(256), 0, s, queries_dev, Q, p.qpad, kb->d, invq, thr64, thrp, cnt, flag, stats, (uint64_t)p.sample_keys, qmask_dev, qmask_pad, p.grid, fb_done);
        else
            hipLaunchKernelGGL(prep_kernel<KB_BF16>, dim3(grid), dim3(256), 0, s, queries_dev, Q, p.qpad, kb->d, invq, thr64, thrp, cnt, flag, stats, (uint64_t)p.sample_keys, qmask_dev, qmask_pad, p.grid, fb_done);
        if (hipGetLastError() != hipSuccess) return KB_ERR_DEVICE;
    }

    if (kb->n > 0) {
        ScanArgs a;
        a.keys = kb->keys;
        a.inv_norm = kb->inv_norm;
        a.tags = qmask_dev ? kb->tags : nullptr;
        a.queries = queries_dev;
        a.qmask = qmask_dev;
        a.qmask_pad = qmask_pad;
        a.invq = invq;
        a.thr64 = thr64;
        a.thrp = thrp;
        a.samp = samp;
        a.regions = regions;
        a.cand = cand;
        a.cnt = cnt;
        a.stats = stats;
        a.cand_cap = p.cand_cap;
        a.flag = flag;
        a.n_keys = kb->n;
        a.d = kb->d;
        a.Q = Q;
        a.nqb = p.nqb;
        a.qpad = p.qpad;
        a.sample_slots = p.sample_slots;
        a.sample_group_shift = 0;        // groups per tile of the sampling configuration: a power of two
        while (p.sample_tiles > 0 && ((int64_t)p.sample_tiles << (a.sample_group_shift + 1)) <= p.sample_slots) ++a.sample_group_shift;
        a.region_cap = p.region_cap;
        a.draw = dr;
        a.tile_stride = 1;
        a.row_mul = 0;
        a.row_run_shift = 0;
        a.row_inv_runs = 0.0;
        a.row_ratio = 0.f;
        if (p.sample_tiles > 0) {
            // the sample is spread evenly over the knowledge base: a prefix says nothing about later rows when
            // the rows are grouped (by state, by cluster, by age)
            a.n_tiles = p.sample_tiles;
            a.tile_stride = (int32_t)(ceil_div(kb->n, p.sample_tk) / p.sample_tiles);
            // ... row by row where the kernel can gather (the two-phase and register-tile kernels load whole tiles:
            // they take every tile_stride-th tile instead)
            a.row_run_shift = draw ? 2 : 0;
            a.row_mul = (p.sample_family == 0 || p.sample_family == 3 || p.sample_family == 4) ? scatter_multiplier(kb->n >> a.row_run_shift) : 0;
            // (the full-line kernel addresses scattered rows in 32 bits, in units of 16 bytes: up to 64 GiB of keys)
            if (p.sample_family == 4 && (uint64_t)kb->n * kb->d * key_bytes(kb->dtype) >= ((uint64_t)1 << 36)) a.row_mul = 0;
            const int64_t runs = (kb->n >> a.row_run_shift) > 0 ? (kb->n >> a.row_run_shift) : 1;
            a.row_inv_runs = 1.0 / (double)runs;
            a.row_ratio = (float)((double)a.row_mul / (double)runs);
            int64_t sgrid = p.sample_tiles * p.nqb;
            const int64_t smax = (int64_t)DEVICE_CUS * p.sample_wgpc;
            if (sgrid > smax && p.sample_family != 4) sgrid = smax;        // (the full-line kernel samples one item per workgroup)
            if (launch_scan(kb->dtype, p.sample_config, p.sample_family, true, (int)sgrid, a, s) != hipSuccess) return KB_ERR_DEVICE;
            const int thr_threads = p.sample_slots > 1024 ? 1024 : p.sample_slots > 512 ? 512 : 256;
            const size_t thr_lds = sizeof(uint64_t) * (p.sample_slots > k ? p.sample_slots : k) + sizeof(SelectScratch);
            ThresholdArgs t;
            t.samp = samp;
            t.queries = queries_dev;
            t.qmask = qmask_dev;
            t.invq = invq;
            t.thrp = thrp;
            t.thr64 = thr64;
            t.qmask_pad = qmask_pad;
            t.stats = stats;
            t.cnt = cnt;
            t.flag = flag;
            t.fb_done = fb_done;
            t.sample_keys = (uint64_t)p.sample_keys;
            t.slots = p.sample_slots;
            t.group_shift = a.sample_group_shift;
            t.k = k;
            t.Q = Q;
            t.qpad = p.qpad;
            t.d = kb->d;
            t.grid = p.grid;
            static LdsAllowed thr_allowed[4];
            const int thr_kind = draw ? 3 : (int)q_dtype;
            void (*thr_fn)(ThresholdArgs) = draw ? &threshold_kernel<KB_F32, true>
                                          : q_dtype == KB_F32 ? &threshold_kernel<KB_F32, false>
                                          : q_dtype == KB_BF16 ? &threshold_kernel<KB_BF16, false> : &threshold_kernel<KB_FP8_E4M3, false>;
            if (allow_dynamic_lds(reinterpret_cast<const void *>(thr_fn), thr_allowed[thr_kind], MAX_SAMPLE_SLOTS * 8 + sizeof(SelectScratch)) != hipSuccess)
                return KB_ERR_DEVICE;
            hipLaunchKernelGGL(thr_fn, dim3(draw ? Q : p.qpad), dim3(thr_threads), thr_lds, s, t);
            if (hipGetLastError() != hipSuccess) return KB_ERR_DEVICE;
        }
        a.n_tiles = ceil_div(kb->n, p.tk);
        a.tile_stride = 1;
        a.row_mul = 0;
        const bool timed = kb->prof_events && kb->prof_used < kb->prof_max && kb->prof_seen++ % kb->prof_stride == kb->prof_stride / 2;
        if (timed) {
            scan_timing.start = kb->prof_events[2 * kb->prof_used];
            scan_timing.stop = kb->prof_events[2 * kb->prof_used + 1];
        }
        const hipError_t launched = launch_scan(kb->dtype, p.config, p.family, false, p.grid, a, s);
        scan_timing = ScanTiming();
        if (launched != hipSuccess) return KB_ERR_DEVICE;
        if (timed) ++kb->prof_used;
    }

    FinalArgs f;
    f.keys = kb->keys;
    f.inv_norm = kb->inv_norm;
    f.tags = qmask_dev ? kb->tags : nullptr;
    f.queries = queries_dev;
    f.qmask = qmask_dev;
    f.invq = invq;
    f.cand = cand;
    f.cnt = cnt;
    f.flag = flag;
    f.stats = stats;
    f.out_index = indices_out_dev;
    f.out_score = scores_out_dev;
    f.n_keys = kb->n;
    f.d = kb->d;
    f.k = k;
    f.cand_cap = p.cand_cap;
    f.draw = dr;
    f.fb_done = fb_done;
    f.fb_lists = reinterpret_cast<uint64_t *>(ws + p.off_fb_lists);
    f.fb_parts = p.fb_parts;
    f.thr64 = thr64;
    f.raw = draw ? 0 : 1;
    const size_t fin_lds = (size_t)p.cand_cap * 8 + 16 + sizeof(SelectScratch);
    static LdsAllowed fin_allowed[4];
    const int fin_kind = q8 ? KT_FP8_Q8 : (int)kb->dtype;
    const void *fin_fn = fin_kind == KB_F32 ? reinterpret_cast<const void *>(&finalize_kernel<KB_F32>)
                       : fin_kind == KB_BF16 ? reinterpret_cast<const void *>(&finalize_kernel<KB_BF16>)
                       : fin_kind == KB_FP8_E4M3 ? reinterpret_cast<const void *>(&finalize_kernel<KB_FP8_E4M3>)
                                                 : reinterpret_cast<const void *>(&finalize_kernel<KT_FP8_Q8>);
    if (allow_dynamic_lds(fin_fn, fin_allowed[fin_kind], MAX_CAND_CAP * 8 + 16 + sizeof(SelectScratch)) != hipSuccess) return KB_ERR_DEVICE;
    switch (fin_kind) {
    case KB_F32: hipLaunchKernelGGL(finalize_kernel<KB_F32>, dim3(Q, p.fb_parts), dim3(256), fin_lds, s, f); break;
    case KB_BF16: hipLaunchKernelGGL(finalize_kernel<KB_BF16>, dim3(Q, p.fb_parts), dim3(256), fin_lds, s, f); break;
    case KB_FP8_E4M3: hipLaunchKernelGGL(finalize_kernel<KB_FP8_E4M3>, dim3(Q, p.fb_parts), dim3(256), fin_lds, s, f); break;
    default: hipLaunchKernelGGL(finalize_kernel<KT_FP8_Q8>, dim3(Q, p.fb_parts), dim3(256), fin_lds, s, f); break;
    }
    if (hipGetLastError() != hipSuccess) return KB_ERR_DEVICE;
    return KB_OK;
}

kb_status_t kb_query(kb_t *kb, const void *queries_dev, kb_dtype_t q_dtype, int32_t Q, const uint64_t *qmask_dev, int32_t k,
                     int32_t *indices_out_dev, float *scores_out_dev, void *workspace_dev, size_t workspace_bytes,
                     void *hip_stream)
{
    return run_query(kb, queries_dev, q_dtype, Q, qmask_dev, k, nullptr, 1.0f, 0, 0, indices_out_dev, scores_out_dev, workspace_dev,
                     workspace_bytes, hip_stream);
}

// The library's own scratch memory for kb_query_static: one array per device, in device memory for as long as the
// process lives.  In host code the name `scratch` only stands for the symbol; its device address is asked for once
// per device (hipGetSymbolAddress, with that device current) and kept in scratch_address[].
static __device__ __align__(256) unsigned char scratch[KB_STATIC_SCRATCH_BYTES];
constexpr int MAX_DEVICES = 64;
static std::atomic<void *> scratch_address[MAX_DEVICES];

kb_status_t kb_query_static(kb_t *kb, const void *queries_dev, kb_dtype_t q_dtype, int32_t Q, const uint64_t *qmask_dev, int32_t k,
                            int32_t *indices_out_dev, float *scores_out_dev, void *hip_stream)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return KB_ERR_DEVICE;
    void *ptr = scratch_address[dev].load(std::memory_order_acquire);
    if (!ptr) {     // first call on this device (two threads racing here get the same address)
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return KB_ERR_DEVICE;
        scratch_address[dev].store(ptr, std::memory_order_release);
    }
    // run_query checks the plan of this call against the size of the array and returns KB_ERR_WORKSPACE beyond it
    return run_query(kb, queries_dev, q_dtype, Q, qmask_dev, k, nullptr, 1.0f, 0, 0, indices_out_dev, scores_out_dev, ptr,
                     KB_STATIC_SCRATCH_BYTES, hip_stream);
}

kb_status_t kb_query_sampled(kb_t *kb, const void *queries_dev, kb_dtype_t q_dtype, int32_t Q, const uint64_t *qmask_dev, int32_t k,
                             const float *gain_dev, float temperature, uint64_t seed, int32_t first_query,
                             int32_t *indices_out_dev, float *keys_out_dev, void *workspace_dev, size_t workspace_bytes,
                             void *hip_stream)
{
    if (!gain_dev) return KB_ERR_NULL;
    if (!(temperature > 0.0f) || !(temperature < __builtin_inff()) || first_query < 0) return KB_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(gain_dev) & 3) != 0) return KB_ERR_INVALID_ARG;
    return run_query(kb, queries_dev, q_dtype, Q, qmask_dev, k, gain_dev, temperature, seed, first_query, indices_out_dev, keys_out_dev,
                     workspace_dev, workspace_bytes, hip_stream);
}

size_t kb_query_probe_workspace_bytes(const kb_t *kb, int32_t Q, int32_t k, int32_t nprobe)
{
    ProbePlan p;
    return kb && make_probe_plan(Q, k, nprobe, &p) ? p.total : 0;
}

kb_status_t kb_query_probe(kb_t *kb, const void *queries_dev, kb_dtype_t q_dtype, int32_t Q, const uint64_t *qmask_dev, int32_t k,
                           const int64_t *cluster_offsets_dev, int32_t n_clusters, const int32_t *probe_dev, int32_t nprobe,
                           int32_t *indices_out_dev, float *scores_out_dev, void *workspace_dev, size_t workspace_bytes, void *hip_stream)
{
    if (!kb || !queries_dev || !cluster_offsets_dev || !probe_dev || !indices_out_dev || !scores_out_dev) return KB_ERR_NULL;
    if (!valid_dtype((int)q_dtype)) return KB_ERR_DTYPE;
    const kb_dtype_t want_q = kb->dtype == KB_F32 ? KB_F32 : KB_BF16;
    const bool q8 = kb->dtype == KB_FP8_E4M3 && q_dtype == KB_FP8_E4M3;
    if (q_dtype != want_q && !q8) return KB_ERR_DTYPE;
    ProbePlan p;
    if (n_clusters < 1 || !make_probe_plan(Q, k, nprobe, &p)) return KB_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(queries_dev) & 15) != 0 || (reinterpret_cast<uintptr_t>(cluster_offsets_dev) & 7) != 0 ||
        (reinterpret_cast<uintptr_t>(probe_dev) & 3) != 0)
        return KB_ERR_INVALID_ARG;
    if (qmask_dev && !kb->tags) return KB_ERR_NO_TAGS;
    if (kb->n_normalized != kb->n) return KB_ERR_NOT_NORMALIZED;
    if (!workspace_dev || (reinterpret_cast<uintptr_t>(workspace_dev) & (WS_ALIGN - 1)) != 0 || workspace_bytes < p.total) return KB_ERR_WORKSPACE;

    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    unsigned char *ws = static_cast<unsigned char *>(workspace_dev);
    float *invq = reinterpret_cast<float *>(ws + p.off_invq);
    uint64_t *lists = reinterpret_cast<uint64_t *>(ws + p.off_lists);
    return launch_probe(kb, false, queries_dev, q_dtype, q8, Q, qmask_dev, k, cluster_offsets_dev, n_clusters, probe_dev, nprobe, p.splits, invq, lists, nullptr,
                        indices_out_dev, scores_out_dev, s);
}

kb_status_t kb_query_counters(const kb_t *kb, const void *workspace_dev, int64_t *out, void *hip_stream)
{
    if (!kb || !workspace_dev || !out) return KB_ERR_NULL;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    if (hipStreamSynchronize(s) != hipSuccess) return KB_ERR_DEVICE;
    uint64_t host[STAT_WORDS + STAT_PARTIALS];
    if (hipMemcpy(host, workspace_dev, sizeof host, hipMemcpyDeviceToHost) != hipSuccess) return KB_ERR_DEVICE;
    for (int i = 0; i < STAT_WORDS; ++i) out[i] = (int64_t)host[i];
    for (int i = 0; i < STAT_PARTIALS; ++i) out[0] += (int64_t)host[STAT_WORDS + i];
    return KB_OK;
}

namespace {
// out[0]: values m of the generator word's upper 23 bits whose variate is below that of m - 1; out[1]: values looked at
__global__ __launch_bounds__(256) void draw_noise_check_kernel(unsigned long long *out)
{
    const uint32_t m = blockIdx.x * 256u + threadIdx.x;      // < 2^23
    const bool falls = m > 0 && gumbel_of_word(m << 9) < gumbel_of_word((m - 1) << 9);
    const unsigned long long bad = __builtin_amdgcn_ballot_w64(falls);
    if ((threadIdx.x & 63) == 0) {
        if (bad) atomicAdd(out, (unsigned long long)__builtin_popcountll(bad));
        atomicAdd(out + 1, 64ull);
    }
}
__global__ void zero_words_kernel(unsigned long long *out, int n)
{
    if ((int)threadIdx.x < n) out[threadIdx.x] = 0ull;
}
}  // namespace

kb_status_t kb_check_draw_noise(int64_t *out_dev, void *hip_stream)
{
    if (!out_dev) return KB_ERR_NULL;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    unsigned long long *out = reinterpret_cast<unsigned long long *>(out_dev);
    hipLaunchKernelGGL(zero_words_kernel, dim3(1), dim3(64), 0, s, out, 2);
    hipLaunchKernelGGL(draw_noise_check_kernel, dim3((1u << 23) / 256), dim3(256), 0, s, out);
    return hipGetLastError() == hipSuccess ? KB_OK : KB_ERR_DEVICE;
}

kb_status_t kb_set_tuning(kb_t *kb, const char *name, int64_t value)
{
    if (!kb || !name) return KB_ERR_NULL;
    if (value < 0) return KB_ERR_INVALID_ARG;
    if (!strcmp(name, "sample_keys")) kb->tune_sample_keys = value;
    else if (!strcmp(name, "scan_config")) {
        ConfigInfo ci;
        if (value != 0 && !scan_config_info(kb->dtype, (int)value, &ci)) return KB_ERR_INVALID_ARG;
        kb->tune_config = value;
    } else if (!strcmp(name, "small_path")) {
        if (value > 1) return KB_ERR_INVALID_ARG;
        kb->tune_no_small_path = value == 0;
    } else if (!strcmp(name, "profile_stride")) {       // of a profiling session, every value-th scan launch is timed, the middle one of each run of `value` (0 = every one)
        kb->prof_stride = value > 0 ? (int)value : 1;
    } else if (!strcmp(name, "wg_per_cu")) {
        if (value > 8) return KB_ERR_INVALID_ARG;
        kb->tune_wg_per_cu = value;
    } else
        return KB_ERR_INVALID_ARG;
    return KB_OK;
}

static void drop_events(kb_t *kb)
{
    if (kb->prof_events) {
        for (int i = 0; i < 2 * kb->prof_max; ++i)
            if (kb->prof_events[i]) (void)hipEventDestroy(kb->prof_events[i]);
        free(kb->prof_events);
    }
    kb->prof_events = nullptr;
    kb->prof_max = kb->prof_used = 0;
}

kb_status_t kb_profile_begin(kb_t *kb, int32_t max_calls)
{
    if (!kb) return KB_ERR_NULL;
    if (max_calls < 1 || max_calls > 4096) return KB_ERR_INVALID_ARG;
    drop_events(kb);
    kb->prof_events = static_cast<hipEvent_t *>(calloc(2 * (size_t)max_calls, sizeof(hipEvent_t)));
    if (!kb->prof_events) return KB_ERR_INVALID_ARG;
    kb->prof_max = max_calls;
    kb->prof_seen = 0;
    for (int i = 0; i < 2 * max_calls; ++i)
        if (hipEventCreate(&kb->prof_events[i]) != hipSuccess) {
            drop_events(kb);
            return KB_ERR_DEVICE;
        }
    return KB_OK;
}

kb_status_t kb_profile_end(kb_t *kb, void *hip_stream, double *scan_ms_total, int32_t *calls)
{
    if (!kb || !scan_ms_total || !calls) return KB_ERR_NULL;
    if (!kb->prof_events) return KB_ERR_INVALID_ARG;
    kb_status_t st = KB_OK;
    if (hipStreamSynchronize(static_cast<hipStream_t>(hip_stream)) != hipSuccess) st = KB_ERR_DEVICE;
    double total = 0.0;
    for (int i = 0; st == KB_OK && i < kb->prof_used; ++i) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, kb->prof_events[2 * i], kb->prof_events[2 * i + 1]) != hipSuccess) st = KB_ERR_DEVICE;
        total += ms;
    }
    *scan_ms_total = total;
    *calls = kb->prof_used;
    drop_events(kb);
    return st;
}

int64_t kb_size(const kb_t *kb) { return kb ? kb->n : -1; }

kb_status_t kb_destroy(kb_t *kb)
{
    if (!kb) return KB_ERR_NULL;
    drop_events(kb);
    delete kb;
    return KB_OK;
}

const char *kb_status_string(kb_status_t s)
{
    switch (s) {
    case KB_OK: return "ok";
    case KB_ERR_NULL: return "required pointer is NULL";
    case KB_ERR_INVALID_ARG: return "argument out of range";
    case KB_ERR_DTYPE: return "dtype not supported for this call";
    case KB_ERR_CAPACITY: return "capacity exceeded";
    case KB_ERR_NOT_NORMALIZED: return "appended rows have not been normalized";
    case KB_ERR_NO_TAGS: return "query mask given for an untagged knowledge base";
    case KB_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case KB_ERR_DEVICE: return "HIP call or kernel launch failed";
    }
    return "unknown status";
}

}  // extern "C"
