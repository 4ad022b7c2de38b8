// Epilogues shared by the scan kernels: what happens to a wave's accumulator blocks once an item's
// contraction is complete.  In the 32x32 accumulator layout lane (lrow, half) of a block holds query
// column lrow and key rows 8*(i/4) + 4*half + (i%4), i = 0..15.
#pragma once
#include "kb_internal.hpp"

namespace kbi {

struct EpiSide {               // side data of the item, in LDS
    const float *invk;         // [TK]  1/|k| of the tile's rows
    const uint64_t *tag;       // [TK]
    const float *thrp;         // [TQ]  pre-filter on dot * inv_k
    const float *invq;         // [TQ]
    const uint64_t *thr64;     // [TQ]  candidate words below this cannot be in the result
    const uint64_t *qmask;     // [TQ]
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
// collected with one v_alignbit each).  Survivors are rare, so the wave then walks them with a
// wave-uniform element index: it takes the mask of one lane that has work (v_readlane), and for each of
// its set bits every lane with that bit handles that element: final score, candidate word, threshold
// word, tag predicate, append to the wave's private record region (no atomics: slot = the wave's running
// count + the lane's rank among the appending lanes; flush_records moves a full region to the per-query
// lists).  A uniform index turns the element selection into an indexed register read instead of a 16-way
// select per lane.
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

__device__ inline void main_block(const f32x16 &a, const EpiRows &rw, float tp, int ql, const EpiSide &sd, bool filter,
                                  int64_t row0, int q0, const ScanArgs &p, Record *region, uint32_t &wave_cnt, uint32_t region_id)
{
    float amax = a[0];
#pragma unroll
    for (int i = 1; i < 16; ++i) amax = __builtin_fmaxf(amax, a[i]);
    // some element can reach the pre-filter only if amax * ikmax does (thrp > 0); otherwise look closer
    const bool maybe = !(__builtin_fmaf(amax, rw.ikmax, -tp) < 0.f) || !(tp > 0.f);
    if (__builtin_amdgcn_ballot_w64(maybe) == 0) return;
    uint32_t fail = 0;
    if (maybe) {
#pragma unroll
        for (int i = 0; i < 16; ++i)
            fail = __builtin_amdgcn_alignbit(fail, as_u32(__builtin_fmaf(a[i], rw.ik[i], -tp)), 31);
    }
    uint32_t pass = maybe ? (~fail & 0xffffu) : 0u;     // element i sits at bit 15 - i
    uint64_t lanes = __builtin_amdgcn_ballot_w64(pass != 0);
    if (lanes == 0) return;
    const float iq = sd.invq[ql];
    const uint64_t t64 = sd.thr64[ql];
    const uint64_t qm = filter ? sd.qmask[ql] : 0ull;
    do {
        // the elements one of the lanes wants looked at; every lane that wants any of them joins in
        uint32_t m = (uint32_t)__builtin_amdgcn_readlane((int)pass, __builtin_ctzll(lanes));
        const uint32_t mine = pass & m;
        pass &= ~m;
        do {
            const int b = 31 - __builtin_clz(m);
            m &= ~(1u << b);
            const int i = 15 - b;                               // wave-uniform
            const bool has = (mine >> b) & 1u;
            const int rl = rw.rl0 + 8 * (i >> 2) + (i & 3);
            const int64_t row = row0 + rl;
            const float ik = sd.invk[rl];
            const uint64_t tg = filter ? sd.tag[rl] : 0ull;    // read with ik: one LDS round trip per element, not two
            const float s = final_score(a[i], ik, iq);
            const uint64_t cw = pack_candidate(s, (uint32_t)row);
            bool ok = has && row < p.n_keys && cw >= t64 && !row_removed(ik);
            if (filter) ok = ok && (tg & qm) != 0;
            // slot in the wave's own record region: running count + rank among the lanes that append (up to 64 of
            // them: the region is emptied first when fewer slots are left)
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
        } while (m != 0);
        lanes = __builtin_amdgcn_ballot_w64(pass != 0);
    } while (lanes != 0);
}

template <int IB, int JB>
__device__ inline void main_epilogue(const f32x16 (&acc)[IB][JB], const EpiSide &sd, bool filter, int wave_row0, int ql0,
                                     int half, int64_t row0, int q0, const ScanArgs &p, Record *region, uint32_t &wave_cnt, uint32_t region_id)
{
    float thrp[JB];
#pragma unroll
    for (int jb = 0; jb < JB; ++jb) thrp[jb] = sd.thrp[ql0 + jb * 32];
#pragma unroll
    for (int ib = 0; ib < IB; ++ib) {
        const EpiRows rw = load_rows(sd, wave_row0 + ib * 32 + 4 * half);
#pragma unroll
        for (int jb = 0; jb < JB; ++jb)
            main_block(acc[ib][jb], rw, thrp[jb], ql0 + jb * 32, sd, filter, row0, q0, p, region, wave_cnt, region_id);
    }
}

// Sampling pass: per lane and query column, one qualifying entry of the lane's rows with the largest
// s1 = dot * inv_k (first one on ties), stored as the candidate word of s1.  The final score is a
// non-decreasing function of s1 (one more fp32 product with 1/|q| >= 0), which the threshold kernel applies:
// the sampling pass itself needs no per-query value but the mask word.  Any qualifying entry is a valid sample.
__device__ inline void sample_block(const f32x16 &a, int rl0, const EpiSide &sd, bool filter, uint64_t qm, int64_t row0,
                                    int64_t n_keys, float &best, int &best_rl)
{
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int rl = rl0 + 8 * (i >> 2) + (i & 3);
        const float ik = sd.invk[rl];
        const float s1 = a[i] * ik;
        bool ok = row0 + rl < n_keys && s1 > best && !row_removed(ik);
        if (filter) ok = ok && (sd.tag[rl] & qm) != 0;
        if (ok) {
            best = s1;
            best_rl = rl;
        }
    }
}

__device__ inline void sample_store(float best, int best_rl, int ql, const EpiSide &sd, int64_t row0, int q0, const ScanArgs &p,
                                    int64_t slot)
{
    if (q0 + ql < p.Q) {
        uint64_t cw = 0ull;
        if (best_rl >= 0)       // best = dot * inv_k was computed exactly as final_score's first product
            cw = pack_candidate(best, sample_index(p, row0 + best_rl));
        p.samp[(size_t)(q0 + ql) * p.sample_slots + slot] = cw;
    }
}

template <int IB, int JB>
__device__ inline void sample_epilogue(const f32x16 (&acc)[IB][JB], const EpiSide &sd, bool filter, int wave_row0, int ql0,
                                       int half, int64_t row0, int q0, const ScanArgs &p, int64_t slot)
{
#pragma unroll
    for (int jb = 0; jb < JB; ++jb) {
        float best = -__builtin_inff();
        int best_rl = -1;
        const uint64_t qm = filter ? sd.qmask[ql0 + jb * 32] : 0ull;
#pragma unroll
        for (int ib = 0; ib < IB; ++ib)
            sample_block(acc[ib][jb], wave_row0 + ib * 32 + 4 * half, sd, filter, qm, row0, p.n_keys, best, best_rl);
        sample_store(best, best_rl, ql0 + jb * 32, sd, row0, q0, p, slot);
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
__device__ inline float gumbel_of_word(uint32_t w)
{
    const float u = __builtin_fmaf((float)(w >> 9), 0x1p-23f, 0x1p-24f);
    return -__logf(-__logf(u));
}

// Key of one (query, entry) pair.  Entries 4j .. 4j+3 share one generator call (counter (j, query, 0, 0)); the word
// is picked by entry % 4.  "+ 0.0f" as in final_score: equal keys have equal bit patterns.
__device__ inline float draw_key(float score, float log_gain, float gumbel, float inv_t)
{
    return (__builtin_fmaf(score, inv_t, log_gain) + gumbel) + 0.0f;
}
__device__ inline float draw_key_of(float score, const DrawArgs &dr, uint32_t query, int64_t row)
{
    uint32_t w[4];
    philox4x32_10((uint32_t)(row >> 2), query, dr.seed_lo, dr.seed_hi, w);
    const uint32_t word = (row & 3) == 0 ? w[0] : (row & 3) == 1 ? w[1] : (row & 3) == 2 ? w[2] : w[3];
    return draw_key(score, dr.log_gain[row], gumbel_of_word(word), dr.inv_t);
}

// Keys of the 16 elements a lane holds in one block (four runs of four consecutive rows: four generator calls).
// SAMPLED: the rows are those of a sampling pass (row0 counts sample rows; runs of four map to their place in the
// knowledge base).
template <bool SAMPLED>
__device__ inline void block_keys(const f32x16 &a, const EpiRows &rw, float iq, const ScanArgs &p, uint32_t query, int64_t row0,
                                  float (&key)[16])
{
    const DrawArgs &dr = p.draw;
#pragma unroll
    for (int run = 0; run < 4; ++run) {
        const int64_t logical = row0 + rw.rl0 + 8 * run;       // a multiple of 4
        const int64_t first = SAMPLED ? (int64_t)sample_index(p, logical) : logical;
        uint32_t w[4];
        philox4x32_10((uint32_t)(first >> 2), query, dr.seed_lo, dr.seed_hi, w);
        const f32x4 lg = *reinterpret_cast<const f32x4 *>(dr.log_gain + first);
        const float lgs[4] = {lg.x, lg.y, lg.z, lg.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int i = 4 * run + e;
            key[i] = draw_key(final_score(a[i], rw.ik[i], iq), lgs[e], gumbel_of_word(w[e]), dr.inv_t);
        }
    }
}

// Main pass on keys.  There is no cheap bound on a key (the noise is unbounded), so every element's key is
// computed and compared with the query's threshold key; survivors are then handled exactly like the survivors
// of the score pass (their keys are recomputed: same inputs, same bits).
__device__ inline void main_block_draw(const f32x16 &a, const EpiRows &rw, float tp, int ql, const EpiSide &sd, bool filter,
                                       int64_t row0, int q0, const ScanArgs &p, Record *region, uint32_t &wave_cnt, uint32_t region_id)
{
    const float iq = sd.invq[ql];
    const uint32_t query = p.draw.first_query + (uint32_t)(q0 + ql);
    float key[16];
    block_keys<false>(a, rw, iq, p, query, row0, key);
    uint32_t pass = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) pass = (pass << 1) | (key[i] >= tp && key[i] > -__builtin_inff() ? 1u : 0u);   // element i at bit 15 - i
    uint64_t lanes = __builtin_amdgcn_ballot_w64(pass != 0);
    if (lanes == 0) return;
    const uint64_t t64 = sd.thr64[ql];
    const uint64_t qm = filter ? sd.qmask[ql] : 0ull;
    do {
        uint32_t m = (uint32_t)__builtin_amdgcn_readlane((int)pass, __builtin_ctzll(lanes));
        const uint32_t mine = pass & m;
        pass &= ~m;
        do {
            const int b = 31 - __builtin_clz(m);
            m &= ~(1u << b);
            const int i = 15 - b;                               // wave-uniform
            const bool has = (mine >> b) & 1u;
            const int rl = rw.rl0 + 8 * (i >> 2) + (i & 3);
            const int64_t row = row0 + rl;
            const float ik = sd.invk[rl];
            const float kv = draw_key_of(final_score(a[i], ik, iq), p.draw, query, row);
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
        } while (m != 0);
        lanes = __builtin_amdgcn_ballot_w64(pass != 0);
    } while (lanes != 0);
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

// Sampling pass on keys: per lane and query column the qualifying entry with the largest key.
template <int IB, int JB>
__device__ inline void sample_epilogue_draw(const f32x16 (&acc)[IB][JB], const EpiSide &sd, bool filter, int wave_row0, int ql0,
                                            int half, int64_t row0, int q0, const ScanArgs &p, int64_t slot)
{
#pragma unroll
    for (int jb = 0; jb < JB; ++jb) {
        const int ql = ql0 + jb * 32;
        const float iq = sd.invq[ql];
        const uint64_t qm = filter ? sd.qmask[ql] : 0ull;
        const uint32_t query = p.draw.first_query + (uint32_t)(q0 + ql);
        float best = -__builtin_inff();
        int best_rl = -1;
#pragma unroll
        for (int ib = 0; ib < IB; ++ib) {
            const EpiRows rw = load_rows(sd, wave_row0 + ib * 32 + 4 * half);
            float key[16];
            block_keys<true>(acc[ib][jb], rw, iq, p, query, row0, key);
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
            p.samp[(size_t)(q0 + ql) * p.sample_slots + slot] = best_rl >= 0 ? pack_candidate(best, sample_index(p, row0 + best_rl)) : 0ull;
    }
}

}  // namespace kbi
