// Epilogues shared by the scan kernels: what happens to a wave's accumulator blocks once an item's
// contraction is complete.  In the 32x32 accumulator layout lane (lrow, half) of a block holds query
// column lrow and key rows 8*(i/4) + 4*half + (i%4), i = 0..15.
#pragma once
#include "kb_internal.hpp"
#include <utility>

namespace kbi {

struct EpiSide {               // side data of the item, in LDS
    const float *invk;         // [TK]  1/|k| of the tile's rows
    const uint64_t *tag;       // [TK]
    const float *thrp;         // [TQ]  pre-filter on dot * inv_k
    const float *invq;         // [TQ]
    const uint64_t *thr64;     // [TQ]  candidate words below this cannot be in the result (read by the weighted selection only)
    const uint64_t *qmask;     // [TQ]
    const float *lgain = nullptr;   // [TK]  ln(gain) of the tile's rows (weighted random selection only)
};

__device__ inline float select16(const f32x16 &a, int i)
{
    float v = a[0];
#pragma unroll
    for (int e = 1; e < 16; ++e) v = (i == e) ? a[e] : v;
    return v;
}

// The records a wavefront has collected in its private region go to the per-query candidate lists: one lane per
// record claims a slot of the record's (query, segment) with a device-wide atomic and stores the candidate word
// there; a full segment flags the query (it is then resolved exhaustively).  Called when the region is nearly full
// and when the wavefront ends, by all its lanes.  The region was written by this wavefront's own global stores: they
// are waited for, and read back past the vector L1 (agent scope), which may hold lines from an earlier call here.
__device__ inline void flush_records(const ScanArgs &p, Record *region, uint32_t &wave_cnt, uint32_t region_id)
{
    if (wave_cnt == 0) return;
    __builtin_amdgcn_s_waitcnt(0x0070 | 0x0F00);        // vmcnt(0): the stores of the records
    const uint32_t lane = __builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
    const uint32_t seg_cap = (uint32_t)p.cand_cap / CAND_SEGMENTS;
    for (uint32_t i = lane; i < wave_cnt; i += 64) {
        const uint64_t cw = __hip_atomic_load(&region[i].cand, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const uint32_t q = __hip_atomic_load(&region[i].query, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const uint32_t seg = candidate_segment(candidate_index(cw));
        const uint32_t slot = atomicAdd(&p.cnt[q * CAND_SEGMENTS + seg], 1u);
        if (slot < seg_cap)
            p.cand[(size_t)q * p.cand_cap + seg * seg_cap + slot] = cw;
        else
            p.flag[q] = 1u;
    }
    if (lane == 0)
        atomicAdd(reinterpret_cast<unsigned long long *>(p.stats + STAT_WORDS + region_id % STAT_PARTIALS), (unsigned long long)wave_cnt);
    wave_cnt = 0;
}

// Main pass.  Per block: a bound test (largest dot times largest 1/|k| of the lane's 16 rows against the
// query's pre-filter) costs one max-reduction and decides whether any lane has to look closer; lanes that
// do build the 16-bit mask of elements passing the exact pre-filter (sign bit of fma(dot, inv_k, -thrp),
// collected with one v_alignbit each).  Survivors are rare (a handful per wave and item), and a wave spends
// their cost with its matrix core idle, so as little as possible is done for them here: every lane with a
// survivor picks its own element (a 16-way select, no wave-uniform walk and no exchange between lanes), checks
// the tag predicate (the one test that can thin the records out by orders of magnitude), drops removed rows and
// appends (dot * inv_k, row, query) to the wave's private record region (no atomics: slot = the wave's running count +
// the lane's rank among the appending lanes; flush_records moves a full region to the per-query lists).  The
// second product of the final score, the exact threshold test and the ordering are left to the kernel that
// selects from the lists, which needs nothing but the query's 1/|q| for them: the pre-filter admits an element
// whenever its final score can reach the threshold (and almost only then), so the lists hold what they would hold
// after an exact test here.
struct EpiRows {               // 1/|k| of the 16 key rows a lane holds in one 32-row block
    float ik[16];
    float ikmax;
    int rl0;                   // tile-local row of element 0
};

__device__ inline EpiRows load_rows(const EpiSide &sd, int rl0)
{
    EpiRows r;
    const f32x4 ik0 = *reinterpret_cast<const f32x4 *>(sd.invk + rl0);
    const f32x4 ik1 = *reinterpret_cast<const f32x4 *>(sd.invk + rl0 + 8);
    const f32x4 ik2 = *reinterpret_cast<const f32x4 *>(sd.invk + rl0 + 16);
    const f32x4 ik3 = *reinterpret_cast<const f32x4 *>(sd.invk + rl0 + 24);
    const float ik[16] = {ik0.x, ik0.y, ik0.z, ik0.w, ik1.x, ik1.y, ik1.z, ik1.w,
                          ik2.x, ik2.y, ik2.z, ik2.w, ik3.x, ik3.y, ik3.z, ik3.w};
    r.ikmax = ik[0];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        r.ik[i] = ik[i];
        r.ikmax = __builtin_fmaxf(r.ikmax, ik[i]);
    }
    r.rl0 = rl0;
    return r;
}

// EXACT: the block test takes the largest dot * inv_k of the lane's elements itself (16 products) instead of the
// product of the two maxima.  For stores whose rows have norms of one size (normalised bf16 or f32 rows) the
// cheap bound is as good; for fp8 codes, whose norms differ by a factor of two from row to row, it lets nine
// blocks in ten through where two in ten hold a survivor.
template <bool EXACT>
__device__ inline void main_block(const f32x16 &a, const EpiRows &rw, float tp, uint64_t qm, uint32_t query, const EpiSide &sd, bool filter,
                                  int64_t row0, const ScanArgs &p, Record *region, uint32_t &wave_cnt, uint32_t region_id)
{
    bool maybe;
    if constexpr (EXACT) {
        float smax = a[0] * rw.ik[0];
#pragma unroll
        for (int i = 1; i < 16; ++i) smax = __builtin_fmaxf(smax, a[i] * rw.ik[i]);
        maybe = !(smax < tp);       // (the survivors' mask below repeats the products as fused ones: never stricter than this)
    } else {
        float amax = a[0];
#pragma unroll
        for (int i = 1; i < 16; ++i) amax = __builtin_fmaxf(amax, a[i]);
        // some element can reach the pre-filter only if amax * ikmax does (thrp > 0); otherwise look closer
        maybe = !(__builtin_fmaf(amax, rw.ikmax, -tp) < 0.f) || !(tp > 0.f);
    }
    if (__builtin_amdgcn_ballot_w64(maybe) == 0) return;
    uint32_t fail = 0;
    if (maybe) {
#pragma unroll
        for (int i = 0; i < 16; ++i)
            fail = __builtin_amdgcn_alignbit(fail, as_u32(__builtin_fmaf(a[i], rw.ik[i], -tp)), 31);
    }
    uint32_t pass = maybe ? (~fail & 0xffffu) : 0u;     // element i sits at bit 15 - i
    while (__builtin_amdgcn_ballot_w64(pass != 0) != 0) {
        const bool has = pass != 0;
        const int b = 31 - __builtin_clz(has ? pass : 1u);
        pass &= ~(1u << b);
        const int i = 15 - b;
        const int rl = rw.rl0 + 8 * (i >> 2) + (i & 3);
        const uint64_t tg = filter ? sd.tag[rl] : 0ull;         // (in flight during the select)
        const float ikv = sd.invk[rl];
        const float dot = select16(a, i);
        const int64_t row = row0 + rl;
        bool ok = has && row < p.n_keys && !row_removed(ikv);
        if (filter) ok = ok && (tg & qm) != 0;
        // slot in the wave's own record region: running count + rank among the lanes that append (up to 64 of
        // them: the region is emptied first when fewer slots are left)
        const uint64_t okm = __builtin_amdgcn_ballot_w64(ok);
        if (okm != 0 && wave_cnt + 64 > (uint32_t)p.region_cap) flush_records(p, region, wave_cnt, region_id);
        if (ok) {
            const uint32_t pos = wave_cnt + __builtin_amdgcn_mbcnt_hi((uint32_t)(okm >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)okm, 0u));
            Record rec;
            rec.cand = pack_raw_candidate(dot * ikv, (uint32_t)row);       // final_score's first product
            rec.query = query;
            rec.pad = 0;
            region[pos] = rec;
        }
        wave_cnt += (uint32_t)__builtin_popcountll(okm);
    }
}

template <int IB, int JB, bool EXACT = false>
__device__ inline void main_epilogue(const f32x16 (&acc)[IB][JB], const EpiSide &sd, bool filter, int wave_row0, int ql0,
                                     int half, int64_t row0, int q0, const ScanArgs &p, Record *region, uint32_t &wave_cnt, uint32_t region_id)
{
    float thrp[JB];
    uint64_t qm[JB];
#pragma unroll
    for (int jb = 0; jb < JB; ++jb) {
        thrp[jb] = sd.thrp[ql0 + jb * 32];
        qm[jb] = filter ? sd.qmask[ql0 + jb * 32] : 0ull;
    }
#pragma unroll
    for (int ib = 0; ib < IB; ++ib) {
        const EpiRows rw = load_rows(sd, wave_row0 + ib * 32 + 4 * half);
#pragma unroll
        for (int jb = 0; jb < JB; ++jb)
            main_block<EXACT>(acc[ib][jb], rw, thrp[jb], qm[jb], (uint32_t)(q0 + ql0 + jb * 32), sd, filter, row0, p, region, wave_cnt, region_id);
    }
}

// Sampling pass: per lane and query column, one qualifying entry of the lane's rows with (nearly) the largest
// s1 = dot * inv_k, stored as the candidate word of s1.  The final score is a non-decreasing function of s1 (one
// more fp32 product with 1/|q| >= 0), which the threshold kernel applies: the sampling pass itself needs no
// per-query value but the mask word.  Any qualifying entry with its exact s1 is a valid sample.
//
// Every element is looked at here, so the search is kept to a few instructions per element: the bits of s1 are read
// as a signed integer (order_key below), the element's number within the lane (5 bits) replaces its low bits, entries
// that fail the tag filter become the smallest integer, and a running integer maximum leaves the number of an
// element whose s1 is within 2^-18 relative of the largest (when that is not negative); that element's exact s1 is
// then recomputed.  Removed
// rows and the repeated rows of a partial tile are not told apart in the search: when one of them wins, its lane
// records no sample for this group of rows, which is always valid (and rare).  Side data
// of the rows is read as 16-byte pieces, four rows at a time.  (Registers are scarce here, with 128 accumulators
// live, and a spilled register costs these kernels dearly: its reload queues behind the stream loads in flight.)
constexpr int32_t SAMPLE_NONE = (int32_t)0x80000000;
// The integer the search compares: the bits of the float as they are.  Non-negative floats keep their order, every
// negative one lies below them, and among negative ones the order is reversed, which costs nothing: a group whose
// best product is negative then records another of its entries, and any qualifying entry with its exact product is a
// valid sample (only the thresholds of queries with fewer than k positive groups could be lower than necessary).
__device__ inline int32_t order_key(float x) { return (int32_t)as_u32(x); }

// one 32x32 block: the best key of the lane's 16 elements joins `best`
__device__ inline void sample_block(const f32x16 &a, int rl0, int id0, const EpiSide &sd, bool filter, uint32_t qm_lo, uint32_t qm_hi,
                                    int32_t &best)
{
#pragma unroll
    for (int run = 0; run < 4; ++run) {             // four runs of four rows: 16 bytes of 1/|k|, 32 bytes of tags
        const int rl = rl0 + 8 * run;
        const f32x4 ik4 = *reinterpret_cast<const f32x4 *>(sd.invk + rl);
        const float ik[4] = {ik4.x, ik4.y, ik4.z, ik4.w};
        u32x4 tg[2] = {};
        if (filter) {
            tg[0] = *reinterpret_cast<const u32x4 *>(sd.tag + rl);
            tg[1] = *reinterpret_cast<const u32x4 *>(sd.tag + rl + 2);
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int i = 4 * run + e;
            int32_t key = (order_key(a[i] * ik[e]) & ~31) | (id0 + i);
            if (filter) {
                const u32x4 t = tg[e >> 1];
                const uint32_t lo = (e & 1) ? t.z : t.x, hi = (e & 1) ? t.w : t.y;
                key = ((lo & qm_lo) | (hi & qm_hi)) != 0 ? key : SAMPLE_NONE;
            }
            best = key > best ? key : best;
        }
    }
}

// The same search with few registers: four elements at a time, their side data read from LDS when it is needed.  For the kernels that keep a software pipeline's fragments live across the
// epilogue and have no registers to spare: there the version above spills, and loses more than it gains.
__device__ inline void sample_block_lean(const f32x16 &a, int rl0, int id0, const EpiSide &sd, bool filter, uint64_t qm, int32_t &best)
{
#pragma unroll
    for (int run = 0; run < 4; ++run) {         // four runs of four rows: one 16-byte read of 1/|k| each
        const int rl = rl0 + 8 * run;
        const f32x4 ik4 = *reinterpret_cast<const f32x4 *>(sd.invk + rl);
        const float ik[4] = {ik4.x, ik4.y, ik4.z, ik4.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int i = 4 * run + e;
            int32_t key = (order_key(a[i] * ik[e]) & ~31) | (id0 + i);
            if (filter) key = (sd.tag[rl + e] & qm) != 0 ? key : SAMPLE_NONE;
            best = key > best ? key : best;
        }
    }
}

template <int IB, int JB, bool LEAN = false>
__device__ inline void sample_epilogue(const f32x16 (&acc)[IB][JB], const EpiSide &sd, bool filter, int wave_row0, int ql0,
                                       int half, int64_t row0, int q0, const ScanArgs &p, int64_t slot, int64_t tile_run, int tk)
{
    static_assert(IB * 16 <= 32, "element numbers take five bits");
#pragma unroll
    for (int jb = 0; jb < JB; ++jb) {
        const int ql = ql0 + jb * 32;
        const uint64_t qm = filter ? sd.qmask[ql] : 0ull;
        int32_t best = SAMPLE_NONE;
#pragma unroll
        for (int ib = 0; ib < IB; ++ib) {
            // the side data is read again for every column: kept from one column to the next it would take a
            // hundred registers that the kernels with a software pipeline do not have
            asm volatile("" ::: "memory");
            if constexpr (LEAN) sample_block_lean(acc[ib][jb], wave_row0 + ib * 32 + 4 * half, ib * 16, sd, filter, qm, best);
            else sample_block(acc[ib][jb], wave_row0 + ib * 32 + 4 * half, ib * 16, sd, filter, (uint32_t)qm, (uint32_t)(qm >> 32), best);
        }
        if (q0 + ql >= p.Q) continue;
        uint64_t cw = 0ull;
        if (best != SAMPLE_NONE) {
            const int e = best & 31, ib = e >> 4, i = e & 15;
            const int rl = wave_row0 + ib * 32 + 4 * half + 8 * (i >> 2) + (i & 3);
            float dot = select16(acc[0][jb], i);
            if (IB > 1 && ib == 1) dot = select16(acc[IB - 1][jb], i);
            const float ikv = sd.invk[rl];
            // a removed row, or a row past the end of the knowledge base (the repeated last row of a partial tile): no sample
            if (!row_removed(ikv) && row0 + rl < p.n_keys)
                cw = pack_candidate(dot * ikv, sample_index(p, tile_run, row0, tk, rl));     // dot * inv_k exactly as final_score's first product
        }
        p.samp[sample_slot_index(slot, p.sample_group_shift, p.qpad, q0 + ql)] = cw;
    }
}

// ------------------------------------------------------------------------------------------------
// Weighted random selection: the same two epilogues on keys = score / T + ln(gain) + Gumbel noise.
// ------------------------------------------------------------------------------------------------

// Philox4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw, SC'11) on the counter (c0, c1, 0, 0).
__device__ inline void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t k0, uint32_t k1, uint32_t (&out)[4])
{
    uint32_t c2 = 0u, c3 = 0u;
#pragma unroll
    for (int round = 0; round < 10; ++round) {
        if (round > 0) {
            k0 += 0x9E3779B9u;
            k1 += 0xBB67AE85u;
        }
        const uint32_t h0 = __umulhi(0xD2511F53u, c0), l0 = 0xD2511F53u * c0;
        const uint32_t h1 = __umulhi(0xCD9E8D57u, c2), l1 = 0xCD9E8D57u * c2;
        c0 = h1 ^ c1 ^ k0;
        c1 = l1;
        c2 = h0 ^ c3 ^ k1;
        c3 = l0;
    }
    out[0] = c0;
    out[1] = c1;
    out[2] = c2;
    out[3] = c3;
}

// Standard Gumbel variate from one generator word: U = (upper 23 bits + 1/2) / 2^23 (exact in fp32), G = -ln(-ln U).
// Both logarithms are the hardware's base-2 logarithm times ln 2: U and -ln U are normal numbers (2^-24 <= U < 1,
// 6e-8 <= -ln U <= 16.7), so the library logarithm's handling of denormals and its extended-precision product (three
// quarters of this function's instructions) buy nothing.  Over all 2^23 values of U the result is within 1.7e-6 of
// the exact variate and non-decreasing in U.
__device__ inline float gumbel_of_word(uint32_t w)
{
    constexpr float LN2 = 0.6931471805599453f;
    const float u = __builtin_fmaf((float)(w >> 9), 0x1p-23f, 0x1p-24f);
    const float l1 = __builtin_amdgcn_logf(u) * LN2;
    return -(__builtin_amdgcn_logf(-l1) * LN2);
}

// Key of one (query, entry) pair.  Entries 4j .. 4j+3 share one generator call (counter (j, query, 0, 0)); the word
// is picked by entry % 4.  "+ 0.0f" as in final_score: equal keys have equal bit patterns.
__device__ inline float draw_key(float score, float log_gain, float gumbel, float inv_t)
{
    return (__builtin_fmaf(score, inv_t, log_gain) + gumbel) + 0.0f;
}
__device__ inline float draw_key_of(float score, float log_gain, const DrawArgs &dr, uint32_t query, int64_t row)
{
    uint32_t w[4];
    philox4x32_10((uint32_t)(row >> 2), query, dr.seed_lo, dr.seed_hi, w);
    const uint32_t word = (row & 3) == 0 ? w[0] : (row & 3) == 1 ? w[1] : (row & 3) == 2 ? w[2] : w[3];
    return draw_key(score, log_gain, gumbel_of_word(word), dr.inv_t);
}
__device__ inline float draw_key_of(float score, const DrawArgs &dr, uint32_t query, int64_t row)
{
    return draw_key_of(score, dr.log_gain[row], dr, query, row);
}

// Keys of the 16 elements a lane holds in one block (four runs of four consecutive rows: four generator calls).
// SAMPLED: the rows are those of a sampling pass (row0 counts sample rows; runs of four map to their place in the
// knowledge base).
template <bool SAMPLED>
__device__ inline void block_keys(const f32x16 &a, const EpiRows &rw, float iq, const ScanArgs &p, uint32_t query, int64_t row0,
                                  const EpiSide &sd, float (&key)[16], int64_t tile_run = 0, int tk = 0)
{
    const DrawArgs &dr = p.draw;
#pragma unroll
    for (int run = 0; run < 4; ++run) {
        const int64_t logical = row0 + rw.rl0 + 8 * run;       // a multiple of 4
        const int64_t first = SAMPLED ? (int64_t)sample_index(p, tile_run, row0, tk, rw.rl0 + 8 * run) : logical;
        uint32_t w[4];
        philox4x32_10((uint32_t)(first >> 2), query, dr.seed_lo, dr.seed_hi, w);
        const f32x4 lg = *reinterpret_cast<const f32x4 *>(sd.lgain + rw.rl0 + 8 * run);
        const float lgs[4] = {lg.x, lg.y, lg.z, lg.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int i = 4 * run + e;
            key[i] = draw_key(final_score(a[i], rw.ik[i], iq), lgs[e], gumbel_of_word(w[e]), dr.inv_t);
        }
    }
}

// The largest generator word (its upper 23 bits, as an integer) with which an element whose noise-free part is at
// most xmax still has a key below the threshold key tp; -1 if there is none.  The noise is a non-decreasing function
// of those bits and the two additions of draw_key are monotone, so every element of the block with bits at or below
// the returned value fails "key >= tp" however its own key rounds.  The value is found from the inverse of the
// Gumbel transform with a margin (fast exponentials, 2 % on the inner one, two steps on the integer) and then checked
// with the very operations of draw_key; a value that fails the check is replaced by a more careful one, then by -1.
__device__ inline int noise_floor(float xmax, float tp)
{
    if (!(tp > -__builtin_inff())) return -1;
    float t = __expf(xmax - tp) * 1.02f;       // e^-c, c = the noise an element at xmax needs
    int m = -1;
#pragma unroll 1
    for (int attempt = 0; attempt < 2; ++attempt) {
        const float mf = __builtin_fmaf(__expf(-t), 0x1p23f, -2.0f);
        const int cand = mf >= 0.f ? (int)__builtin_fminf(mf, 8388607.f) : -1;
        if (cand < 0) break;
        const float key = (xmax + gumbel_of_word((uint32_t)cand << 9)) + 0.0f;
        if (key < tp) {
            m = cand;
            break;
        }
        t *= 8.f;
    }
    return m;
}

// Main pass on keys.  Computing a key costs a generator call per four elements and two logarithms per element; the
// test against the query's threshold key does not need them: with the largest noise-free part of the lane's 16
// elements, noise_floor gives the generator word below which no element of the block can pass, and the per-element
// test is one integer compare on the generator's output.  What passes (the elements whose key can reach the
// threshold, and as many again) is handled like the survivors of the score pass, each lane walking its own
// elements, with the exact key and the exact tests.
__device__ inline void main_block_draw(const f32x16 &a, const EpiRows &rw, float tp, int ql, const EpiSide &sd, bool filter,
                                       int64_t row0, int q0, const ScanArgs &p, Record *region, uint32_t &wave_cnt, uint32_t region_id)
{
    const DrawArgs &dr = p.draw;
    const float iq = sd.invq[ql];
    const uint32_t query = dr.first_query + (uint32_t)(q0 + ql);
    float xmax = -__builtin_inff();
#pragma unroll
    for (int run = 0; run < 4; ++run) {
        const f32x4 lg = *reinterpret_cast<const f32x4 *>(sd.lgain + rw.rl0 + 8 * run);
        const float lgs[4] = {lg.x, lg.y, lg.z, lg.w};
#pragma unroll
        for (int e = 0; e < 4; ++e)
            xmax = __builtin_fmaxf(xmax, __builtin_fmaf(final_score(a[4 * run + e], rw.ik[4 * run + e], iq), dr.inv_t, lgs[e]));
    }
    const int floor_m = noise_floor(xmax, tp);
    const uint32_t floor_w = floor_m < 0 ? 0u : ((uint32_t)floor_m << 9) | 0x1ffu;
    uint32_t pass = 0;
#pragma unroll
    for (int run = 0; run < 4; ++run) {
        uint32_t w[4];
        philox4x32_10((uint32_t)((row0 + rw.rl0 + 8 * run) >> 2), query, dr.seed_lo, dr.seed_hi, w);
#pragma unroll
        for (int e = 0; e < 4; ++e) pass = (pass << 1) | (w[e] > floor_w ? 1u : 0u);       // element i at bit 15 - i
    }
    if (floor_m < 0) pass = 0xffffu;
    if (__builtin_amdgcn_ballot_w64(pass != 0) == 0) return;
    const uint64_t t64 = sd.thr64[ql];
    const uint64_t qm = filter ? sd.qmask[ql] : 0ull;
    do {
        const bool has = pass != 0;
        const int b = 31 - __builtin_clz(has ? pass : 1u);
        pass &= ~(1u << b);
        const int i = 15 - b;
        const int rl = rw.rl0 + 8 * (i >> 2) + (i & 3);
        const int64_t row = row0 + rl;
        const float ik = sd.invk[rl];
        const float kv = draw_key_of(final_score(select16(a, i), ik, iq), sd.lgain[rl], dr, query, row);
        const uint64_t cw = pack_candidate(kv, (uint32_t)row);
        bool ok = has && row < p.n_keys && kv > -__builtin_inff() && cw >= t64 && !row_removed(ik);
        if (filter) ok = ok && (sd.tag[rl] & qm) != 0;
        const uint64_t okm = __builtin_amdgcn_ballot_w64(ok);
        if (okm != 0 && wave_cnt + 64 > (uint32_t)p.region_cap) flush_records(p, region, wave_cnt, region_id);
        if (ok) {
            const uint32_t pos = wave_cnt + __builtin_amdgcn_mbcnt_hi((uint32_t)(okm >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)okm, 0u));
            Record rec;
            rec.cand = cw;
            rec.query = (uint32_t)(q0 + ql);
            rec.pad = 0;
            region[pos] = rec;
        }
        wave_cnt += (uint32_t)__builtin_popcountll(okm);
    } while (__builtin_amdgcn_ballot_w64(pass != 0) != 0);
}

template <int IB, int JB>
__device__ inline void main_epilogue_draw(const f32x16 (&acc)[IB][JB], const EpiSide &sd, bool filter, int wave_row0, int ql0,
                                          int half, int64_t row0, int q0, const ScanArgs &p, Record *region, uint32_t &wave_cnt, uint32_t region_id)
{
#pragma unroll
    for (int ib = 0; ib < IB; ++ib) {
        const EpiRows rw = load_rows(sd, wave_row0 + ib * 32 + 4 * half);
#pragma unroll
        for (int jb = 0; jb < JB; ++jb)
            main_block_draw(acc[ib][jb], rw, sd.thrp[ql0 + jb * 32], ql0 + jb * 32, sd, filter, row0, q0, p, region, wave_cnt, region_id);
    }
}

// Sampling pass on keys: per lane and query column the qualifying entry with the largest key.  One function per
// query column of the wave's tile, expanded at compile time: as a loop over the columns the body (eight generator
// calls and 32 keys per column) is too large to be unrolled, and the accumulators, indexed by a loop counter, would
// live in scratch memory.
template <int IB, int JB, int JBX>
__device__ inline void sample_column_draw(const f32x16 (&acc)[IB][JB], const EpiSide &sd, bool filter, int wave_row0, int ql0,
                                          int half, int64_t row0, int q0, const ScanArgs &p, int64_t slot, int64_t tile_run, int tk)
{
    const int ql = ql0 + JBX * 32;
    const float iq = sd.invq[ql];
    const uint64_t qm = filter ? sd.qmask[ql] : 0ull;
    const uint32_t query = p.draw.first_query + (uint32_t)(q0 + ql);
    float best = -__builtin_inff();
    int best_rl = -1;
#pragma unroll
    for (int ib = 0; ib < IB; ++ib) {
        // (the row number is opaque per block: otherwise the side data and the scattered-row arithmetic of all the
        // wave's rows, which do not depend on the column, are kept in registers across the columns and spilled)
        int rl0 = wave_row0 + ib * 32 + 4 * half;
        asm volatile("" : "+v"(rl0));
        const EpiRows rw = load_rows(sd, rl0);
        float key[16];
        block_keys<true>(acc[ib][JBX], rw, iq, p, query, row0, sd, key, tile_run, tk);
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int rl = rw.rl0 + 8 * (i >> 2) + (i & 3);
            bool ok = row0 + rl < p.n_keys && key[i] > best && !row_removed(rw.ik[i]);
            if (filter) ok = ok && (sd.tag[rl] & qm) != 0;
            if (ok) {
                best = key[i];
                best_rl = rl;
            }
        }
    }
    if (q0 + ql < p.Q)
        p.samp[sample_slot_index(slot, p.sample_group_shift, p.qpad, q0 + ql)] = best_rl >= 0 ? pack_candidate(best, sample_index(p, tile_run, row0, tk, best_rl)) : 0ull;
}

template <int IB, int JB, int... JBX>
__device__ inline void sample_columns_draw(const f32x16 (&acc)[IB][JB], const EpiSide &sd, bool filter, int wave_row0, int ql0, int half, int64_t row0,
                                           int q0, const ScanArgs &p, int64_t slot, int64_t tile_run, int tk, std::integer_sequence<int, JBX...>)
{
    (sample_column_draw<IB, JB, JBX>(acc, sd, filter, wave_row0, ql0, half, row0, q0, p, slot, tile_run, tk), ...);
}

template <int IB, int JB>
__device__ inline void sample_epilogue_draw(const f32x16 (&acc)[IB][JB], const EpiSide &sd, bool filter, int wave_row0, int ql0,
                                            int half, int64_t row0, int q0, const ScanArgs &p, int64_t slot, int64_t tile_run, int tk)
{
    sample_columns_draw<IB, JB>(acc, sd, filter, wave_row0, ql0, half, row0, q0, p, slot, tile_run, tk, std::make_integer_sequence<int, JB>{});
}

}  // namespace kbi
