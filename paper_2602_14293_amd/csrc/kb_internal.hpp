// Internal declarations shared by the translation units of libkb (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include <atomic>

#include "kb.h"

// The handle: host-side bookkeeping over caller-owned device storage.
struct kb {
    int32_t d;
    kb_dtype_t dtype;
    int64_t capacity, n, n_normalized;
    void *keys;
    float *row_scale, *inv_norm;
    uint64_t *tags;
    int64_t tune_sample_keys, tune_config, tune_wg_per_cu, tune_no_small_path;
    hipEvent_t *prof_events;   // 2 * prof_max events while profiling, else nullptr
    int prof_max, prof_used;
    int prof_stride, prof_seen;   // every prof_stride-th scan launch of a profiling session is timed
};

namespace kbi {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

// Bit reinterpretation of scalars passed BY VALUE.  (__builtin_bit_cast applied directly to a vector
// element such as v[e] or f.y has been seen to read element 0 instead; never do that.)
__host__ __device__ inline float as_f32(uint32_t x) { return __builtin_bit_cast(float, x); }
__host__ __device__ inline uint32_t as_u32(float x) { return __builtin_bit_cast(uint32_t, x); }

// A candidate is one 64-bit sortable word: larger word = earlier in the result order
// (score descending, index ascending).  0 is never a valid candidate ("empty").
//   high 32 bits: the fp32 score mapped monotonically onto unsigned integers
//   low  32 bits: ~index  (index < 2^31, so a smaller index gives a larger word)
__host__ __device__ inline uint32_t score_to_ordered(float s)
{
    uint32_t u = __builtin_bit_cast(uint32_t, s);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__host__ __device__ inline float ordered_to_score(uint32_t o)
{
    uint32_t u = (o & 0x80000000u) ? (o & 0x7fffffffu) : ~o;
    return __builtin_bit_cast(float, u);
}
__host__ __device__ inline uint64_t pack_candidate(float score, uint32_t index)
{
    return ((uint64_t)score_to_ordered(score) << 32) | (uint32_t)(~index);
}
__host__ __device__ inline uint32_t candidate_index(uint64_t c) { return ~(uint32_t)c; }
// What the main pass of a scan leaves in the candidate lists of a plain query: the bits of dot * inv_k (the first
// product of final_score) instead of the ordered score, which the kernel that selects from the lists derives with the
// query's 1/|q|; the same low word.
__host__ __device__ inline uint64_t pack_raw_candidate(float dot_inv_k, uint32_t index)
{
    return ((uint64_t)__builtin_bit_cast(uint32_t, dot_inv_k) << 32) | (uint32_t)(~index);
}
__host__ __device__ inline float raw_candidate_product(uint64_t c) { return __builtin_bit_cast(float, (uint32_t)(c >> 32)); }
__host__ __device__ inline float candidate_score(uint64_t c) { return ordered_to_score((uint32_t)(c >> 32)); }

// The fp32 score every kernel of the library computes from an fp32 dot product.
// "+ 0.0f" turns -0.0 into +0.0 so that equal scores have equal bit patterns.
__device__ inline float final_score(float dot, float inv_k, float inv_q) { return (dot * inv_k) * inv_q + 0.0f; }

// A removed entry keeps its row and its index but is never a candidate again: kb_remove sets the sign bit of its
// 1/|k| (which is never negative otherwise; a zero row's 0 becomes -0).
constexpr uint32_t REMOVED_BIT = 0x80000000u;
__host__ __device__ inline bool row_removed(float inv_k) { return (as_u32(inv_k) & REMOVED_BIT) != 0; }

// Kernel-side name of "fp8 keys with fp8 queries" where a kernel template is selected by key type: the keys are
// KB_FP8_E4M3 either way, but both operands go to the fp8 matrix instruction as they are stored.
constexpr int KB_FP8_Q8 = 3;

struct Record {  // one candidate that passed the threshold filter of the scan
    uint64_t cand;
    uint32_t query;
    uint32_t pad;
};

// A query's candidate list is CAND_SEGMENTS segments with a counter each, so that the slot-claiming atomics of one
// query are spread over that many addresses instead of serialising on one.  A candidate's segment comes from its
// row number: a query's candidates spread over all segments even when they sit in a few neighbouring tiles (rows
// grouped by cluster) and were found by a few workgroups; consecutive rows take the segments in turn.
constexpr int CAND_SEGMENTS = 16;
__host__ __device__ inline uint32_t candidate_segment(uint32_t row) { return (row ^ (row >> 4) ^ (row >> 8)) % CAND_SEGMENTS; }
// Diagnostics at the start of the workspace: STAT_WORDS words (candidates, exhaustive queries, sample keys, scan
// workgroups), then the candidate count as STAT_PARTIALS partial sums (one hot address would serialise).
constexpr int STAT_WORDS = 4;
constexpr int STAT_PARTIALS = 64;
// Records a scan wavefront collects before it moves them to the per-query lists (it also does so when it ends).
constexpr int REGION_CAP = 128;

// Workspace layout (offsets in bytes from a 256-byte aligned base).
struct Plan {
    int32_t Q, k, tq, nqb, qpad;        // queries, tile width in queries, query blocks, padded count
    int32_t config;                     // scan tile configuration id
    int family;                         // which kernel family the configuration belongs to (ConfigInfo::family)
    int32_t tk;                         // keys per tile
    int32_t groups_per_tile;            // sample groups per key tile
    int32_t sample_config, sample_family, sample_wgpc, sample_tk;   // the sampling pass may use another scan configuration (and tile height)
    int64_t sample_tiles;               // key tiles (of the sampling configuration) scored by the sampling pass (0 = none)
    int64_t sample_keys;                // rows they cover
    int32_t sample_slots;               // sample_tiles * groups_per_tile, per query
    int32_t grid;                       // workgroups of the main scan
    int32_t region_cap;                 // records a scan wavefront collects before it moves them to the lists
    int32_t regions;                    // grid * wavefronts per workgroup
    int32_t cand_cap;                   // candidates per query the final sort can take (power of two)
    size_t off_fb_done, off_fb_lists;       // exhaustive path: per-query arrival counters, per-(query, part) partial lists
    int32_t fb_parts;                      // parts the rows are split into when a query takes the exhaustive path
    size_t off_invq, off_thr64, off_thrp, off_cnt, off_flag, off_stats, off_qmask, off_samp, off_regions,
        off_cand, off_lgain, total;
};

// Weighted random selection (Section 3, Optimization Selector: its top-k is a random draw whose weights are the
// entries' predicted gains): entries are ranked by key = score / T + ln(gain) + Gumbel noise instead of by
// score, which draws k entries without replacement with probability proportional to gain * exp(score / T).
struct DrawArgs {
    const float *log_gain;    // [rows padded to a multiple of 256]: ln(gain), -inf for entries that are never drawn
    float inv_t;              // 1 / temperature
    uint32_t seed_lo, seed_hi;
    uint32_t first_query;     // the noise of query row r is that of global query number first_query + r
    int32_t enabled;
};

struct ScanArgs {
    const void *keys;
    const float *inv_norm;
    const uint64_t *tags;     // nullptr when no filter is applied
    const void *queries;
    const uint64_t *qmask;    // nullptr when no filter is applied
    const uint64_t *qmask_pad; // [qpad] copy of qmask padded with zero words (library workspace)
    const float *invq;        // [qpad]
    const uint64_t *thr64;    // [qpad] candidate words below this cannot be in the result
    const float *thrp;        // [qpad] conservative pre-filter on dot * inv_k
    uint64_t *samp;           // sampling pass output [sample tiles][qpad][groups per tile]: see sample_slot_index
    Record *regions;          // [grid * waves per workgroup][region_cap]: one private region per wavefront
    uint64_t *cand;           // [qpad][cand_cap] per-query candidate lists, CAND_SEGMENTS segments each
    uint32_t *cnt;            // [qpad][CAND_SEGMENTS] entries claimed in each segment (zero before the launch)
    uint32_t *flag;           // [qpad] set to 1 when a query lost a candidate to a full list
    uint64_t *stats;          // diagnostics (see STAT_WORDS)
    int64_t n_keys;           // rows to scan: [0, n_keys)
    int64_t n_tiles;          // key tiles to scan: logical tile t is rows [t * tile_stride * TK, +TK)
    int32_t tile_stride;      // 1 for the main pass; a sampling pass takes every tile_stride-th tile ...
    uint64_t row_mul;         // ... or, when nonzero, scatters its rows in runs of 2^row_run_shift (see sample_row)
    double row_inv_runs;      // 1 / (n_keys >> row_run_shift)
    float row_ratio;          // row_mul / (n_keys >> row_run_shift)
    int32_t row_run_shift;
    int32_t d, Q, nqb, qpad, sample_slots, sample_group_shift, region_cap, cand_cap;
    DrawArgs draw;
};

// Key row behind row r of logical tile `tile` in a sampling pass.  With row_mul the sample is scattered in runs of
// R = 2^row_run_shift rows: run j of the sample is run (j * row_mul) mod (n_keys / R) of the knowledge base (row_mul
// coprime to the number of runs and about 0.618 of it: one to one, consecutive runs far apart).  Every group of
// rows whose maximum the sampling epilogue keeps then mixes rows from all over the knowledge base, so the
// threshold stays tight when the rows are grouped by cluster.  R = 1 for the plain retrieval; the weighted
// selection takes runs of four, which keep what it shares between neighbouring rows (one generator call, one
// 16-byte load of gains).  Without row_mul the tile is tile_stride tiles further on and rows past the end repeat
// the last row.
//
// The map is linear, so a workgroup maps the first run of its tile once (sample_tile_run: exact 64-bit arithmetic with
// a quotient estimated in double precision; a 64-bit division would be a software routine of some hundred
// instructions) and every row of the tile from that (sample_row: the product of a run number below 256 with row_mul
// has a quotient below 256, which single precision estimates to within one).
__device__ inline int64_t mulmod_runs(const ScanArgs &p, int64_t run)      // (run * row_mul) mod runs, run < runs < 2^31
{
    const int64_t runs = p.n_keys >> p.row_run_shift, prod = run * (int64_t)p.row_mul;
    int64_t r = prod - (int64_t)((double)prod * p.row_inv_runs) * runs;
    r += r < 0 ? runs : 0;
    r -= r >= runs ? runs : 0;
    return r;
}
__device__ inline int64_t sample_tile_run(const ScanArgs &p, int64_t tile, int tk)     // mapped run of the tile's first row
{
    return p.row_mul ? mulmod_runs(p, (tile * tk) >> p.row_run_shift) : 0;
}
__device__ inline int64_t sample_row(const ScanArgs &p, int64_t tile_run, int64_t tile, int tk, int r)     // 0 <= r < tk <= 256
{
    if (p.row_mul) {
        const int sh = p.row_run_shift;
        const int64_t runs = p.n_keys >> sh;
        const uint32_t lr = (uint32_t)r >> sh;                                          // run within the tile
        const uint32_t q = (uint32_t)((float)lr * p.row_ratio);                         // floor(lr * row_mul / runs), or one off
        int64_t m = (int64_t)((uint64_t)lr * p.row_mul) - (int64_t)((uint64_t)q * (uint64_t)runs);
        m += m < 0 ? runs : 0;
        m -= m >= runs ? runs : 0;
        m += tile_run;
        m -= m >= runs ? runs : 0;
        return (m << sh) + (r & ((1 << sh) - 1));
    }
    const int64_t row = tile * p.tile_stride * tk + r;
    return row < p.n_keys ? row : p.n_keys - 1;
}
// first row number the sampling epilogues count from: logical when the rows are scattered
__device__ inline int64_t sample_row0(const ScanArgs &p, int64_t tile, int tk) { return p.row_mul ? tile * tk : tile * p.tile_stride * tk; }
// knowledge-base row of tile-local row rl of a sampling pass whose epilogue counts rows from row0 = sample_row0()
__device__ inline uint32_t sample_index(const ScanArgs &p, int64_t tile_run, int64_t row0, int tk, int rl)
{
    return (uint32_t)(p.row_mul ? sample_row(p, tile_run, 0, tk, rl) : row0 + rl);
}

// Where sample `slot` (= tile * groups + group) of query q lives.  The groups of one tile are adjacent (64 bytes per
// query for eight groups) and the queries of a tile follow each other: a sampling wavefront stores words 64 bytes apart
// inside one 16 KiB run instead of 16 KiB apart, and the threshold kernel reads a query's samples 64 bytes at a time.
__host__ __device__ inline size_t sample_slot_index(int64_t slot, int group_shift, int qpad, int q)      // groups = 2^group_shift
{
    return ((((size_t)slot >> group_shift) * qpad + q) << group_shift) + ((size_t)slot & ((1u << group_shift) - 1));
}

// A kernel that uses more than 64 KiB of dynamic LDS must be allowed to, once per device (the attribute belongs to the
// device's copy of the kernel).  `done` holds one bit per device ordinal; callers keep one such word per kernel.
// Two threads that race here both set the attribute, which is harmless.
typedef std::atomic<uint64_t> LdsAllowed;
inline hipError_t allow_dynamic_lds(const void *kernel, LdsAllowed &done, size_t bytes)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const uint64_t bit = (dev >= 0 && dev < 64) ? 1ull << dev : 0ull;       // beyond 64 devices: set it on every call
    if (bit && (done.load(std::memory_order_acquire) & bit)) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e == hipSuccess && bit) done.fetch_or(bit, std::memory_order_release);
    return e;
}

// Kernel timing for roofline reports (kb_profile_begin): while `start` is set, the next scan launch of this thread
// carries the two events on its own dispatch packet (hipExtLaunchKernelGGL), so that their difference is the
// kernel's duration and no extra packets sit between it and its neighbours (events recorded around a launch cost
// about 7 us each).
struct ScanTiming {
    hipEvent_t start = nullptr, stop = nullptr;
};
extern thread_local ScanTiming scan_timing;

// Launchers, one translation unit per key dtype.  `sample` selects the sampling epilogue.
hipError_t launch_scan_f32(int config, bool sample, int grid, const ScanArgs &a, hipStream_t s);
hipError_t launch_scan_bf16(int config, bool sample, int grid, const ScanArgs &a, hipStream_t s);
hipError_t launch_scan_fp8(int config, bool sample, int grid, const ScanArgs &a, hipStream_t s);
hipError_t launch_scan_sp_bf16(int config, bool sample, int grid, const ScanArgs &a, hipStream_t s);
hipError_t launch_scan_wide_bf16(int config, bool sample, int grid, const ScanArgs &a, hipStream_t s);
hipError_t launch_scan_wide_fp8(int config, bool sample, int grid, const ScanArgs &a, hipStream_t s);
hipError_t launch_scan_sp_fp8(int config, bool sample, int grid, const ScanArgs &a, hipStream_t s);

// Static description of a scan configuration (host side planning).
struct ConfigInfo {
    int tk, tq, threads, groups_per_tile, wg_per_cu;
    int min_row_bytes;      // smallest key row (bytes) the configuration's pipeline is valid for
    int family;             // 0: kb_scan.hpp, 3: kb_scan_sp.hpp, 4: kb_scan_wide.hpp
};
bool scan_config_info(int key_dtype, int config, ConfigInfo *out);   // false if the id does not exist
int scan_config_for(int key_dtype, int Q, int d, int64_t n);         // automatic choice for n rows

}  // namespace kbi
