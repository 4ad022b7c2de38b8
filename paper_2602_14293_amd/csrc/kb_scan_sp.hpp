// The large-batch scan kernel, software-pipelined variant: 8 wavefronts, 256 key rows x 256 queries per work
// item, 64-byte row pieces; a wavefront reads its operand fragments from LDS *between its MFMAs* instead of
// in a phase of their own, and there is ONE workgroup barrier per d-chunk (gfx950 only).
//
// A d-chunk (64 bytes of every key row) is two k-groups of 32 bytes.  Fragments live in two register
// sets, X (k-group 0) and Y (k-group 1); while the MFMAs of one set run, the other set is refilled:
//
//   compute part of chunk g:   8 MFMAs on X = kg0(g)   with the 6 reads  Y <- kg1(g)    in between,
//                              8 MFMAs on Y = kg1(g)   with the 6 reads  X <- kg0(g+1)  in between
//   load part of chunk g:      epilogue of a finished item, then this wave's share of the direct-to-LDS
//                              loads of chunk g + NS - 1 (NS = ring depth)
//
// Between two barriers every wave runs both parts, waves 0-3 compute first, waves 4-7 load first.  Each
// SIMD hosts one wave of either kind, so its matrix core is fed by one wave while the other issues loads
// (a direct-to-LDS load holds the issuing wave for tens of cycles) or runs an epilogue, and nothing but
// the one barrier forces the two to move in step.  Iteration g reads chunks g and g+1 only, and its
// loads overwrite the ring slot of chunk g-1, which nobody touches after barrier g.  A wave arrives at
// barrier g+1 once its share of chunk g+2 has landed (NS-3 younger chunks still in flight).  Key chunks
// come from HBM and get a ring of 5, query chunks come from L2 and get 4.
//
// IL mode (256-query blocks of bf16 x bf16 and of fp8 x fp8): no split into compute-first and load-first
// waves.  Every wave issues its share of the direct-to-LDS loads of chunk g + NS - 1 *between the MFMAs* of
// chunk g (one load after every fourth bf16 MFMA, after every second fp8 MFMA), then waits, meets the one
// barrier, and runs a finished item's epilogue after it.  A wave held in the issue of a direct-to-LDS load
// does not leave its SIMD's matrix core to the other wave as well as a wave with MFMAs in flight does
// (probe: 16 MFMAs + 4 loads per wave and chunk take 0.46 ms interleaved, 0.49 ms in two phases, 0.50 ms
// split).  Measured gain over the split: 2-3 % on 2^20 x 1024 bf16 keys with 256 queries, 5 % on 2^22 x 768
// fp8 keys with 1024 fp8 queries; fp8 keys with bf16 queries (32 MFMAs per chunk) gain nothing and keep it.
//
// LDS layout of a chunk: 64-byte rows with the XOR swizzle of kb_scan.hpp, 16 rows per
// load instruction (requests of 64 bytes are what the L2 serves best; 32-byte requests cost 1.6x the L2
// requests and 1.25x the HBM traffic when measured).  To make room for the deeper ring, the per-query
// side data has one LDS copy, reloaded in an item's second iteration (every epilogue of the previous item
// is over by then).
#pragma once
#include "kb_scan.hpp"

namespace kbi {

// bytes 0-7 / 8-15 of a 16-byte run of e4m3 codes as eight bf16 values (exact: see e4m3_pair_to_bf16)
__device__ inline u32x4 widen_e4m3_lo(u32x4 a)
{
    return u32x4{e4m3_pair_to_bf16(a.x, false), e4m3_pair_to_bf16(a.x, true), e4m3_pair_to_bf16(a.y, false), e4m3_pair_to_bf16(a.y, true)};
}
__device__ inline u32x4 widen_e4m3_hi(u32x4 a)
{
    return u32x4{e4m3_pair_to_bf16(a.z, false), e4m3_pair_to_bf16(a.z, true), e4m3_pair_to_bf16(a.w, false), e4m3_pair_to_bf16(a.w, true)};
}

template <int KT_, int TQ_, int NSA_, int NSB_, bool QF8_ = false, bool IL_ = false> struct SPCfg {
    static constexpr int KT = KT_, TQ = TQ_, NSA = NSA_, NSB = NSB_;       // query block; ring depths in chunks: keys, queries
    static constexpr bool QF8 = QF8_;                                      // fp8 keys AND fp8 queries: the fp8 matrix instruction
    static constexpr bool IL = IL_;                                        // loads between the MFMAs instead of a load part
    static constexpr int TK = 256, THREADS = 512, NW = 8;
    static constexpr int KEY_BYTES = KeyTraits<KT>::KEY_BYTES, QRY_BYTES = QF8 ? 1 : KeyTraits<KT>::QRY_BYTES;
    static constexpr int BMUL = QRY_BYTES / KEY_BYTES;                     // 2 for fp8 keys with bf16 queries
    static constexpr int RBA = 64, RBB = RBA * BMUL;                       // bytes of a key / query row per chunk
    static constexpr int PPRB = RBB / 16;
    static constexpr int IB = 2, JB = TQ / 2 / 32;
    static constexpr int A_BYTES = TK * RBA, B_BYTES = TQ * RBB;
    static constexpr int LCA = A_BYTES / 1024 / 4, LCB = B_BYTES / 1024 / 4;   // load instructions per loading wave per chunk
    static constexpr int OFF_B = NSA * A_BYTES;
    // side data of a key tile, two copies (item parity)
    static constexpr int AUX_INVK = 0;                       // float  [TK]
    static constexpr int AUX_TAG = AUX_INVK + TK * 4;        // uint64 [TK]
    static constexpr int AUX_BYTES = AUX_TAG + TK * 8;
    // side data of a query block, one copy
    static constexpr int QAUX_THRP = 0;                      // float  [TQ]
    static constexpr int QAUX_INVQ = QAUX_THRP + TQ * 4;     // float  [TQ]
    static constexpr int QAUX_THR64 = QAUX_INVQ + TQ * 4;    // uint64 [TQ]
    static constexpr int QAUX_QMASK = QAUX_THR64 + TQ * 8;   // uint64 [TQ]
    static constexpr int QAUX_BYTES = QAUX_QMASK + TQ * 8;
    static constexpr int OFF_AUX = OFF_B + NSB * B_BYTES;
    static constexpr int OFF_QAUX = OFF_AUX + 2 * AUX_BYTES;
    static constexpr int SMEM_BYTES = OFF_QAUX + QAUX_BYTES;
    static constexpr int GROUPS_PER_TILE = 8;                // sampling groups: 4 row blocks x 2 lane halves
    static constexpr int MIN_ROW_BYTES = RBA * ((NSA > NSB ? NSA : NSB) + 1);   // the side-data buffers alternate safely only then
    static_assert(TQ == 256 || TQ == 128, "query blocks of 256 or 128");
    static_assert((KT == KB_BF16 && BMUL == 1 && !QF8) || (KT == KB_FP8_E4M3 && TQ == 256 && (BMUL == 2 || QF8)), "key types the kernel is written for");
    static_assert(NSA >= 3 && NSA <= 6 && NSB >= 3 && NSB <= 6, "ring depths the waits are written for");
    static_assert(SMEM_BYTES <= 160 * 1024, "LDS budget");
    static_assert(!IL || (TQ == 256 && (KT == KB_BF16 || QF8)), "the interleaved mode is written for 256-query blocks of bf16 x bf16 and fp8 x fp8");
};

template <class C, bool SAMPLE>
__global__ __launch_bounds__(512, 1) void kb_scan_sp_kernel(ScanArgs p)
{
    constexpr int TK = C::TK, TQ = C::TQ, RBA = C::RBA, RBB = C::RBB, IB = C::IB, JB = C::JB, NW = C::NW;
    constexpr int LC = C::LCA > C::LCB ? C::LCA : C::LCB;
    static_assert(IB == 2 && (JB == 4 || JB == 2), "the interleaving below is written out for 2 x 4 and 2 x 2 blocks");
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    typedef __attribute__((address_space(3))) void *lds_ptr;
    // load destinations are kept as 32-bit pointers of the LDS address space: a generic pointer would be converted (with
    // its null check) at every load
    typedef __attribute__((address_space(3))) unsigned char lds_u8;
    lds_u8 *const lds = (lds_u8 *)smem;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave & 3, group = wave >> 2;
    const int lrow = lane & 31, half = lane >> 5;
    const bool filter = p.qmask != nullptr;

    const int nqb = p.nqb;
    const int64_t tstride = p.tile_stride;     // 1, or the distance between the tiles of a sampling pass
    const int64_t n_items = p.n_tiles * nqb;
    const int vb = item_lane(blockIdx.x, gridDim.x, nqb);      // this workgroup takes items vb, vb + gridDim.x, ...
    const int my_items = (int64_t)vb < n_items ? (int)((n_items - vb + gridDim.x - 1) / gridDim.x) : 0;
    const int NC = p.d * C::KEY_BYTES / RBA;
    const int total = my_items * NC;
    const uint32_t key_row_bytes = (uint32_t)p.d * C::KEY_BYTES, qry_row_bytes = (uint32_t)p.d * C::QRY_BYTES;
    const int step_tile = gridDim.x / nqb, step_qb = gridDim.x % nqb;

    Record *my_region = p.regions + ((size_t)blockIdx.x * NW + wave) * p.region_cap;
    uint32_t wave_cnt = 0;       // wave-uniform

    // ---- the load stream of this wave: key chunks (role 0) or query chunks (role 1) -------------------
    // Instruction j of a chunk covers 1 KiB of it: 16 rows of four 16-byte pieces (64-byte rows) or 8 rows of eight.
    const int role = wave & 1, ridx = wave >> 1;
    const int NS = role ? C::NSB : C::NSA;
    const int D = NS - 1;                                   // chunk g+D is issued in iteration g
    const int LCr = role ? C::LCB : C::LCA;                 // this wave's load instructions per chunk
    const int ppr = role ? C::PPRB : 4;                     // 16-byte pieces per row
    const int ld_row = (ridx * 64 + lane) / ppr, ld_rstep = 256 / ppr;
    const uint32_t ld_piece = (uint32_t)(((ridx * 64 + lane) % ppr) ^ (role && C::PPRB == 8 ? swizzle<8>(ld_row) : swizzle<4>(ld_row))) * 16;
    const uint32_t row_bytes = role ? qry_row_bytes : key_row_bytes, chunk_bytes = role ? RBB : RBA;
    const unsigned char *src_base = role ? static_cast<const unsigned char *>(p.queries) : static_cast<const unsigned char *>(p.keys);
    lds_u8 *ring = lds + (role ? C::OFF_B : 0) + ridx * 1024;
    int ld_pos = 0;                                         // chunks issued so far
    int ld_tile = vb / nqb, ld_qb = vb % nqb;
    int ld_c = 0, ld_stage = 0, ld_par = 0;
    typedef typename std::conditional<SAMPLE, uint64_t, uint32_t>::type Off;   // a sampling pass addresses key rows anywhere
    Off off[LC];
    size_t ld_base = 0;                                     // byte offset of the item's first row in the source
    bool last_full = false;
    auto ld_setup = [&]() {
        const int last = role == 0 ? (int)(p.n_keys - ld_tile * tstride * TK < TK ? p.n_keys - ld_tile * tstride * TK - 1 : TK - 1)
                                   : p.Q - 1 - ld_qb * TQ;
        const int64_t tile_run = (SAMPLE && role == 0) ? sample_tile_run(p, ld_tile, TK) : 0;
#pragma unroll
        for (int j = 0; j < LC; ++j) {
            int r = ld_row + j * ld_rstep;
            // (a sampling pass maps r to a scattered row with some 64-bit arithmetic whose first part does not depend on
            // the tile: computed once per lane and load and kept across the items, those values are spilled and each
            // reload waits for every stream load in flight; r is therefore opaque here and the map is computed per tile)
            if constexpr (SAMPLE) asm volatile("" : "+v"(r));
            if (SAMPLE && role == 0) off[j] = (Off)((uint64_t)sample_row(p, tile_run, ld_tile, TK, r) * row_bytes + ld_piece);
            else off[j] = (uint32_t)(r < last ? r : last) * row_bytes + ld_piece;
        }
        ld_base = role == 0 ? (SAMPLE ? 0 : (size_t)(ld_tile * tstride) * TK * row_bytes) : (size_t)ld_qb * TQ * row_bytes;
    };
    // side data of a key tile: 4-byte loads with clamped rows from the caller's arrays
    auto issue_tile_aux = [&]() {
        lds_u8 *aux = lds + C::OFF_AUX + ld_par * C::AUX_BYTES;
        const int64_t row0 = ld_tile * tstride * TK;
        const int64_t tile_run = SAMPLE ? sample_tile_run(p, ld_tile, TK) : 0;
        if (wave < 4) {
            int64_t r = row0 + wave * 64 + lane;
            r = r < p.n_keys ? r : p.n_keys - 1;
            if constexpr (SAMPLE) {
                int rl = wave * 64 + lane;
                asm volatile("" : "+v"(rl));
                r = sample_row(p, tile_run, ld_tile, TK, rl);
            }
            __builtin_amdgcn_global_load_lds((const void *)(p.inv_norm + r), (lds_ptr)(aux + C::AUX_INVK + wave * 256), 4, 0, 0);
        }
        if (filter) {
            // tags as dwords: wave w covers dwords [64w, 64w+64) = rows [32w, 32w+32)
            int64_t r = row0 + wave * 32 + (lane >> 1);
            r = r < p.n_keys ? r : p.n_keys - 1;
            if constexpr (SAMPLE) {
                int rl = wave * 32 + (lane >> 1);
                asm volatile("" : "+v"(rl));
                r = sample_row(p, tile_run, ld_tile, TK, rl);
            }
            __builtin_amdgcn_global_load_lds((const void *)(reinterpret_cast<const uint32_t *>(p.tags + r) + (lane & 1)),
                                             (lds_ptr)(aux + C::AUX_TAG + wave * 256), 4, 0, 0);
        }
    };
    // side data of a query block: 16-byte loads from the library's padded per-query arrays, one array per wave.  A
    // sampling pass runs before those exist and needs the mask words only: it takes them from the caller's array as
    // dwords with clamped query numbers (wave w covers queries [32 w, 32 w + 32), and the next 32 x 8 with 256 queries).
    auto issue_query_aux = [&](int qb) {
        lds_u8 *aux = lds + C::OFF_QAUX;
        const int q0 = qb * TQ;
        if constexpr (SAMPLE) {
            if (filter) {
                const int last = p.Q - 1 - q0;
                for (int i = wave; i < TQ / 32; i += NW) {
                    const int r = i * 32 + (lane >> 1);
                    __builtin_amdgcn_global_load_lds((const void *)(reinterpret_cast<const uint32_t *>(p.qmask + q0 + (r < last ? r : last)) + (lane & 1)),
                                                     (lds_ptr)(aux + C::QAUX_QMASK + i * 256), 4, 0, 0);
                }
            }
            return;
        }
        constexpr int L4 = TQ / 4, W8 = TQ * 8 / 1024;          // lanes that cover a float array; waves that cover a 64-bit array
        if (wave == 0 && lane < L4)
            __builtin_amdgcn_global_load_lds((const void *)(p.invq + q0 + lane * 4), (lds_ptr)(aux + C::QAUX_INVQ), 16, 0, 0);
        if (wave == 1 && lane < L4)
            __builtin_amdgcn_global_load_lds((const void *)(p.thrp + q0 + lane * 4), (lds_ptr)(aux + C::QAUX_THRP), 16, 0, 0);
        if (wave >= 2 && wave < 2 + W8)
            __builtin_amdgcn_global_load_lds((const void *)(p.thr64 + q0 + (wave - 2) * 128 + lane * 2),
                                             (lds_ptr)(aux + C::QAUX_THR64 + (wave - 2) * 1024), 16, 0, 0);
        if (wave >= 4 && wave < 4 + W8 && filter)
            __builtin_amdgcn_global_load_lds((const void *)(p.qmask_pad + q0 + (wave - 4) * 128 + lane * 2),
                                             (lds_ptr)(aux + C::QAUX_QMASK + (wave - 4) * 1024), 16, 0, 0);
    };
    // One load phase's issue: this wave's share of the chunk at the cursor, if any is left.
    auto issue_round = [&]() {
        last_full = ld_pos < total;
        if (!last_full) return;
        if (ld_c == 0) issue_tile_aux();
        const unsigned char *g = src_base + ld_base + (size_t)ld_c * chunk_bytes;
        lds_u8 *dst = ring + ld_stage * (role ? C::B_BYTES : C::A_BYTES);
#pragma unroll
        for (int j = 0; j < LC; ++j)
            if (j < LCr) __builtin_amdgcn_global_load_lds((const void *)(g + off[j]), (lds_ptr)(dst + j * 4096), 16, 0, 0);
        ++ld_pos;
        ld_stage = ld_stage + 1 == NS ? 0 : ld_stage + 1;
        if (++ld_c == NC) {
            ld_c = 0;
            ld_par ^= 1;
            ld_tile += step_tile;
            ld_qb += step_qb;
            if (ld_qb >= nqb) {
                ld_qb -= nqb;
                ++ld_tile;
            }
            if (ld_pos < total) ld_setup();
        }
    };
    // The same round in three steps, for the mode that puts the loads between the MFMAs.
    const unsigned char *il_src = nullptr;
    lds_u8 *il_dst = ring;
    auto issue_prepare = [&]() {
        last_full = ld_pos < total;
        if (!last_full) return;
        if (ld_c == 0) issue_tile_aux();
        il_src = src_base + ld_base + (size_t)ld_c * chunk_bytes;
        il_dst = ring + ld_stage * (role ? C::B_BYTES : C::A_BYTES);
    };
    auto issue_one = [&](int j) {
        if (last_full && j < LCr) __builtin_amdgcn_global_load_lds((const void *)(il_src + off[j]), (lds_ptr)(il_dst + j * 4096), 16, 0, 0);
    };
    auto issue_finish = [&]() {
        if (!last_full) return;
        ++ld_pos;
        ld_stage = ld_stage + 1 == NS ? 0 : ld_stage + 1;
        if (++ld_c == NC) {
            ld_c = 0;
            ld_par ^= 1;
            ld_tile += step_tile;
            ld_qb += step_qb;
            if (ld_qb >= nqb) {
                ld_qb -= nqb;
                ++ld_tile;
            }
            if (ld_pos < total) ld_setup();
        }
    };
    // All but the youngest NS-3 chunks of this wave's stream have landed once at most LCr * (NS-3) loads are
    // outstanding (side-data loads only make the wait longer).  Once the stream has run dry, wait for everything.
    auto wait_landed = [&]() {
        if (!last_full) __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));
        else if (LCr * (NS - 3) == 2) __builtin_amdgcn_s_waitcnt(waitcnt_vm(2));
        else if (LCr * (NS - 3) == 4) __builtin_amdgcn_s_waitcnt(waitcnt_vm(4));
        else if (LCr * (NS - 3) == 6) __builtin_amdgcn_s_waitcnt(waitcnt_vm(6));
        else if (LCr * (NS - 3) == 8) __builtin_amdgcn_s_waitcnt(waitcnt_vm(8));
        else if (LCr * (NS - 3) == 12) __builtin_amdgcn_s_waitcnt(waitcnt_vm(12));
        else __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));
    };

    // ---- fragment addresses ----------------------------------------------------------------------
    const int rowA = wm * 64 + lrow;
    const int rowB = group * (TQ / 2) + lrow;
    const int fragA = rowA * RBA | ((half ^ swizzle<4>(rowA)) << 4);     // ^ (kg << 5), + ib * 32 * RBA
    // query bytes that go with a lane's 16 key bytes: one piece (same element width) or two adjacent ones
    const int fragB = C::BMUL == 1 ? (rowB * RBB | ((half ^ swizzle<4>(rowB)) << 4))
                                   : (rowB * RBB | (((2 * half) ^ swizzle<8>(rowB)) << 4));
    auto read_a = [&](int stage, int kg, int ib) {
        return *reinterpret_cast<const u32x4 *>(smem + stage * C::A_BYTES + ((fragA ^ (kg << 5)) + ib * 32 * RBA));
    };
    auto read_b = [&](int stage, int kg, int jb, int second = 0) {
        return *reinterpret_cast<const u32x4 *>(smem + C::OFF_B + stage * C::B_BYTES +
                                                ((fragB ^ (kg * 32 * C::BMUL) ^ (second << 4)) + jb * 32 * RBB));
    };

    f32x16 acc[IB][JB];
#pragma unroll
    for (int ib = 0; ib < IB; ++ib)
#pragma unroll
        for (int jb = 0; jb < JB; ++jb)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[ib][jb][i] = 0.f;

    auto epilogue = [&](int tile, int qb, int par) {
        // What the epilogue derives from the item's coordinates and from the lane's place in the tile (addresses of
        // its outputs, LDS addresses of the lane's query and rows) is computed here: kept across the chunks it
        // sits in registers the software pipeline needs, gets spilled, and a reload queues behind the stream
        // loads in flight.
        int rowB_e = rowB, half_e = half;
        asm volatile("" : "+s"(tile), "+s"(qb), "+s"(par), "+v"(rowB_e), "+v"(half_e));
        const int rowB = rowB_e, half = half_e;
        const unsigned char *aux = smem + C::OFF_AUX + par * C::AUX_BYTES, *qaux = smem + C::OFF_QAUX;
        const EpiSide sd{reinterpret_cast<const float *>(aux + C::AUX_INVK), reinterpret_cast<const uint64_t *>(aux + C::AUX_TAG),
                         reinterpret_cast<const float *>(qaux + C::QAUX_THRP), reinterpret_cast<const float *>(qaux + C::QAUX_INVQ),
                         reinterpret_cast<const uint64_t *>(qaux + C::QAUX_THR64), reinterpret_cast<const uint64_t *>(qaux + C::QAUX_QMASK)};
        const int64_t row0 = SAMPLE ? sample_row0(p, tile, TK) : tile * tstride * TK;
        if (SAMPLE)
            sample_epilogue<IB, JB, true>(acc, sd, filter, wm * 64, rowB, half, row0, qb * TQ, p,
                                    (int64_t)tile * C::GROUPS_PER_TILE + wm * 2 + half, sample_tile_run(p, tile, TK), TK);
        else
            main_epilogue<IB, JB, C::KEY_BYTES == 1>(acc, sd, filter, wm * 64, rowB, half, row0, qb * TQ, p, my_region, wave_cnt, blockIdx.x * NW + wave);
#pragma unroll
        for (int ib = 0; ib < IB; ++ib)
#pragma unroll
            for (int jb = 0; jb < JB; ++jb)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[ib][jb][i] = 0.f;
    };

    // ---- prologue: chunks 0 .. D-1 issued, chunks 0 and 1 landed, kg0 of chunk 0 read ----------------
    if (total > 0) {
        ld_setup();
        issue_query_aux(vb % nqb);
    }
    for (int s = 0; s < D; ++s) issue_round();
    wait_landed();
    __builtin_amdgcn_s_waitcnt(waitcnt_lgkm0());
    bare_barrier();                         // barrier 0
    u32x4 xa[IB], xb[JB], ya[IB], yb[JB];
    u32x4 ra[IB];                               // fp8 keys: raw fragments of the k-group whose low half is in X
    if constexpr (!C::QF8) {
#pragma unroll
        for (int ib = 0; ib < IB; ++ib) {
            ra[ib] = read_a(0, 0, ib);
            xa[ib] = C::BMUL == 2 ? widen_e4m3_lo(ra[ib]) : ra[ib];
        }
#pragma unroll
        for (int jb = 0; jb < JB; ++jb) xb[jb] = read_b(0, 0, jb);
    }
    if (!C::IL && group == 1) issue_round();    // split mode: waves 4-7 run their load part ahead of the compute part

    int tile = vb / nqb, qb = vb % nqb, par = 0;
    int c = 0, stageA = 0, stageB = 0;
    bool pending = false;                   // an item is complete and waits for its epilogue
    int e_tile = 0, e_qb = 0, e_par = 0;

#define KB_SP_MFMA(SA, SB, I, J)                                                                                            \
    acc[I][J] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, SA[I]), __builtin_bit_cast(bf16x8, SB[J]), \
                                                        acc[I][J], 0, 0, 0);                                                  \
    __builtin_amdgcn_sched_barrier(0)
    // interleaved mode: load j of the round prepared at the top of the iteration
#define KB_SP_LOAD(J)                      \
    if constexpr (C::IL) {                 \
        issue_one(J);                      \
        __builtin_amdgcn_sched_barrier(0); \
    }
    // what follows an iteration's MFMAs: bookkeeping, then (in the order of the wave's kind) barrier and load part
    auto finish_iteration = [&](int c_now, int qb_now) {
        stageA = stageA + 1 == C::NSA ? 0 : stageA + 1;
        stageB = stageB + 1 == C::NSB ? 0 : stageB + 1;
        if (++c == NC) {
            pending = true;
            e_tile = tile;
            e_qb = qb;
            e_par = par;
            c = 0;
            par ^= 1;
            tile += step_tile;
            qb += step_qb;
            if (qb >= nqb) {
                qb -= nqb;
                ++tile;
            }
        }
        if (group == 1) {
            wait_landed();
            __builtin_amdgcn_s_waitcnt(waitcnt_lgkm0());
            __builtin_amdgcn_sched_barrier(0);
            bare_barrier();
            __builtin_amdgcn_sched_barrier(0);
        }
        // load part: of this iteration (waves 0-3) or of the next one (waves 4-7)
        if (pending) {
            epilogue(e_tile, e_qb, e_par);
            pending = false;
        }
        __builtin_amdgcn_sched_barrier(0);
        if (nqb > 1 && (group == 0 ? c_now == 1 : c == 1)) issue_query_aux(group == 0 ? qb_now : qb);
        issue_round();
        __builtin_amdgcn_sched_barrier(0);
        if (group == 0) {
            wait_landed();
            __builtin_amdgcn_s_waitcnt(waitcnt_lgkm0());
            __builtin_amdgcn_sched_barrier(0);
            bare_barrier();
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // interleaved mode: what precedes and what follows an iteration's MFMAs
    auto begin_iteration_il = [&]() {
        if (nqb > 1 && c == 1) issue_query_aux(qb);     // every epilogue of the previous item ended before the last barrier
        issue_prepare();
        __builtin_amdgcn_sched_barrier(0);
    };
    auto finish_iteration_il = [&]() {
        issue_finish();
        stageA = stageA + 1 == C::NSA ? 0 : stageA + 1;
        stageB = stageB + 1 == C::NSB ? 0 : stageB + 1;
        if (++c == NC) {
            pending = true;
            e_tile = tile;
            e_qb = qb;
            e_par = par;
            c = 0;
            par ^= 1;
            tile += step_tile;
            qb += step_qb;
            if (qb >= nqb) {
                qb -= nqb;
                ++tile;
            }
        }
        wait_landed();
        __builtin_amdgcn_s_waitcnt(waitcnt_lgkm0());
        __builtin_amdgcn_sched_barrier(0);
        bare_barrier();
        __builtin_amdgcn_sched_barrier(0);
        if (pending) {
            epilogue(e_tile, e_qb, e_par);
            pending = false;
        }
    };

    if constexpr (!C::QF8) {
        for (int g = 0; g < total; ++g) {
            // Waves 0-3: compute(g), load(g), barrier.  Waves 4-7: [load(g) was done before the previous barrier's
            // successor, see below] compute(g), barrier, load(g+1).  One code path, two barrier positions.
            const int c_now = c, qb_now = qb;
            if constexpr (C::IL) begin_iteration_il();
            {
                const int nA = stageA + 1 == C::NSA ? 0 : stageA + 1, nB = stageB + 1 == C::NSB ? 0 : stageB + 1;
                // past the last chunk the refill of X reads the current slot again (valid memory, values unused)
                const int xA = g + 1 < total ? nA : stageA, xB = g + 1 < total ? nB : stageB;
                __builtin_amdgcn_s_setprio(1);
                if constexpr (C::BMUL == 2) {
                    // fp8 keys: the 16 key bytes a lane holds per k-group widen to two bf16 operands ("lo" = bytes 0-7,
                    // "hi" = bytes 8-15), each paired with its own 16-byte query piece.  A chunk is therefore four steps of
                    // eight MFMAs (kg0 lo, kg0 hi, kg1 lo, kg1 hi: the accumulation order of every other kernel); X serves
                    // the lo steps, Y the hi steps, and each is refilled while the other is in use.  ra holds the raw key
                    // fragments of the k-group whose lo half is in X.
#define KB_SP_8MFMA(SA, SB, R0, R1, R2)                                             \
        KB_SP_MFMA(SA, SB, 0, 0); R0; __builtin_amdgcn_sched_barrier(0);                \
        KB_SP_MFMA(SA, SB, 0, 1); R1; __builtin_amdgcn_sched_barrier(0);                \
        KB_SP_MFMA(SA, SB, 1, 0); R2; __builtin_amdgcn_sched_barrier(0);                \
        KB_SP_MFMA(SA, SB, 1, 1); KB_SP_MFMA(SA, SB, 0, 2); KB_SP_MFMA(SA, SB, 1, 2);   \
        KB_SP_MFMA(SA, SB, 0, 3); KB_SP_MFMA(SA, SB, 1, 3)
                    // kg0 lo; refill Y with kg0 hi
                    KB_SP_8MFMA(xa, xb, (yb[0] = read_b(stageB, 0, 0, 1), yb[1] = read_b(stageB, 0, 1, 1)),
                                (yb[2] = read_b(stageB, 0, 2, 1), yb[3] = read_b(stageB, 0, 3, 1)),
                                (ya[0] = widen_e4m3_hi(ra[0]), ya[1] = widen_e4m3_hi(ra[1])));
                    // kg0 hi; refill X with kg1 lo
                    KB_SP_8MFMA(ya, yb, (ra[0] = read_a(stageA, 1, 0), ra[1] = read_a(stageA, 1, 1)),
                                (xb[0] = read_b(stageB, 1, 0), xb[1] = read_b(stageB, 1, 1)),
                                (xb[2] = read_b(stageB, 1, 2), xb[3] = read_b(stageB, 1, 3)));
                    xa[0] = widen_e4m3_lo(ra[0]);
                    xa[1] = widen_e4m3_lo(ra[1]);
                    __builtin_amdgcn_sched_barrier(0);
                    // kg1 lo; refill Y with kg1 hi
                    KB_SP_8MFMA(xa, xb, (yb[0] = read_b(stageB, 1, 0, 1), yb[1] = read_b(stageB, 1, 1, 1)),
                                (yb[2] = read_b(stageB, 1, 2, 1), yb[3] = read_b(stageB, 1, 3, 1)),
                                (ya[0] = widen_e4m3_hi(ra[0]), ya[1] = widen_e4m3_hi(ra[1])));
                    // kg1 hi; refill X with kg0 lo of the next chunk
                    KB_SP_8MFMA(ya, yb, (ra[0] = read_a(xA, 0, 0), ra[1] = read_a(xA, 0, 1)),
                                (xb[0] = read_b(xB, 0, 0), xb[1] = read_b(xB, 0, 1)),
                                (xb[2] = read_b(xB, 0, 2), xb[3] = read_b(xB, 0, 3)));
                    xa[0] = widen_e4m3_lo(ra[0]);
                    xa[1] = widen_e4m3_lo(ra[1]);
                    __builtin_amdgcn_sched_barrier(0);
#undef KB_SP_8MFMA
                } else if constexpr (JB == 4) {
                // The reads sit behind the first three MFMAs of each half: the remaining five cover their latency, and the
                    // MFMA order lets the next half start on the fragments that were read first.
                    KB_SP_MFMA(xa, xb, 0, 0);
                    ya[0] = read_a(stageA, 1, 0);
                    yb[0] = read_b(stageB, 1, 0);
                    __builtin_amdgcn_sched_barrier(0);
                    KB_SP_MFMA(xa, xb, 0, 1);
                    yb[1] = read_b(stageB, 1, 1);
                    ya[1] = read_a(stageA, 1, 1);
                    __builtin_amdgcn_sched_barrier(0);
                    KB_SP_MFMA(xa, xb, 1, 0);
                    yb[2] = read_b(stageB, 1, 2);
                    yb[3] = read_b(stageB, 1, 3);
                    __builtin_amdgcn_sched_barrier(0);
                    KB_SP_MFMA(xa, xb, 1, 1);
                    KB_SP_LOAD(0);
                    KB_SP_MFMA(xa, xb, 0, 2);
                    KB_SP_MFMA(xa, xb, 1, 2);
                    KB_SP_LOAD(1);
                    KB_SP_MFMA(xa, xb, 0, 3);
                    KB_SP_MFMA(xa, xb, 1, 3);

                    KB_SP_MFMA(ya, yb, 0, 0);
                    xa[0] = read_a(xA, 0, 0);
                    xb[0] = read_b(xB, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
                    KB_SP_MFMA(ya, yb, 0, 1);
                    xb[1] = read_b(xB, 0, 1);
                    xa[1] = read_a(xA, 0, 1);
                    __builtin_amdgcn_sched_barrier(0);
                    KB_SP_MFMA(ya, yb, 1, 0);
                    xb[2] = read_b(xB, 0, 2);
                    xb[3] = read_b(xB, 0, 3);
                    __builtin_amdgcn_sched_barrier(0);
                    KB_SP_MFMA(ya, yb, 1, 1);
                    KB_SP_LOAD(2);
                    KB_SP_MFMA(ya, yb, 0, 2);
                    KB_SP_MFMA(ya, yb, 1, 2);
                    KB_SP_LOAD(3);
                    KB_SP_MFMA(ya, yb, 0, 3);
                    KB_SP_MFMA(ya, yb, 1, 3);
                } else {
                    KB_SP_MFMA(xa, xb, 0, 0);
                    ya[0] = read_a(stageA, 1, 0);
                    yb[0] = read_b(stageB, 1, 0);
                    __builtin_amdgcn_sched_barrier(0);
                    KB_SP_MFMA(xa, xb, 0, 1);
                    yb[1] = read_b(stageB, 1, 1);
                    ya[1] = read_a(stageA, 1, 1);
                    __builtin_amdgcn_sched_barrier(0);
                    KB_SP_MFMA(xa, xb, 1, 0);
                    KB_SP_MFMA(xa, xb, 1, 1);

                    KB_SP_MFMA(ya, yb, 0, 0);
                    xa[0] = read_a(xA, 0, 0);
                    xb[0] = read_b(xB, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
                    KB_SP_MFMA(ya, yb, 0, 1);
                    xb[1] = read_b(xB, 0, 1);
                    xa[1] = read_a(xA, 0, 1);
                    __builtin_amdgcn_sched_barrier(0);
                    KB_SP_MFMA(ya, yb, 1, 0);
                    KB_SP_MFMA(ya, yb, 1, 1);
                }
                __builtin_amdgcn_s_setprio(0);

            }
            if constexpr (C::IL) {
                finish_iteration_il();
            } else {
                finish_iteration(c_now, qb_now);
            }
        }
    } else {
        // fp8 keys and fp8 queries: one v_mfma_f32_32x32x64_f8f6f4 per block and d-chunk (a lane supplies 32 bytes of
        // its row per operand: lane half h owns bytes [32h, 32h+32) of the 64-byte chunk).  Key fragments live in two
        // sets of whole chunks (the set of chunk g+1 is filled while chunk g is computed; the roles swap every
        // iteration, hence two iterations per loop trip).  Query fragments rotate through two buffers instead: the
        // MFMAs run column block by column block, and while block jb is computed the fragment of block jb+1 (or of
        // block 0 of the next chunk) is read.  That keeps the fragments at 48 registers beside the 128 accumulators.
        typedef int i32x8 __attribute__((ext_vector_type(8)));
        typedef int i32x4 __attribute__((ext_vector_type(4)));
        i32x8 fa0[IB], fa1[IB], fq0, fq1;             // .lo = first 16 bytes of the lane's 32, .hi = second
        const int fragA8 = rowA * RBA, fragB8 = rowB * RBB, swzA = swizzle<4>(rowA), swzB = swizzle<4>(rowB);
        auto read_a8 = [&](int stage, int ib, int t) {
            return *reinterpret_cast<const i32x4 *>(smem + stage * C::A_BYTES + fragA8 + ib * 32 * RBA + (((2 * half + t) ^ swzA) << 4));
        };
        auto read_b8 = [&](int stage, int jb, int t) {
            return *reinterpret_cast<const i32x4 *>(smem + C::OFF_B + stage * C::B_BYTES + fragB8 + jb * 32 * RBB + (((2 * half + t) ^ swzB) << 4));
        };
#pragma unroll
        for (int ib = 0; ib < IB; ++ib) {
            fa0[ib].lo = read_a8(0, ib, 0);
            fa0[ib].hi = read_a8(0, ib, 1);
        }
        fq0.lo = read_b8(0, 0, 0);
        fq0.hi = read_b8(0, 0, 1);
        auto iteration8 = [&](int g, const i32x8 (&ca)[IB], i32x8 (&na)[IB]) {
            const int c_now = c, qb_now = qb;
            if constexpr (C::IL) begin_iteration_il();
            const int nA = stageA + 1 == C::NSA ? 0 : stageA + 1, nB = stageB + 1 == C::NSB ? 0 : stageB + 1;
            // past the last chunk the refill reads the current slot again (valid memory, values unused)
            const int xA = g + 1 < total ? nA : stageA, xB = g + 1 < total ? nB : stageB;
            __builtin_amdgcn_s_setprio(1);
#define KB_SP_MFMA8(I, J, FQ)                                                                                      \
    acc[I][J] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(ca[I], FQ, acc[I][J], 0, 0, 0, 0, 0, 0);           \
    __builtin_amdgcn_sched_barrier(0)
            KB_SP_MFMA8(0, 0, fq0);
            fq1.lo = read_b8(stageB, 1, 0);
            fq1.hi = read_b8(stageB, 1, 1);
            __builtin_amdgcn_sched_barrier(0);
            KB_SP_MFMA8(1, 0, fq0);
            KB_SP_LOAD(0);
            na[0].lo = read_a8(xA, 0, 0);
            na[0].hi = read_a8(xA, 0, 1);
            __builtin_amdgcn_sched_barrier(0);
            KB_SP_MFMA8(0, 1, fq1);
            fq0.lo = read_b8(stageB, 2, 0);
            fq0.hi = read_b8(stageB, 2, 1);
            __builtin_amdgcn_sched_barrier(0);
            KB_SP_MFMA8(1, 1, fq1);
            KB_SP_LOAD(1);
            na[1].lo = read_a8(xA, 1, 0);
            na[1].hi = read_a8(xA, 1, 1);
            __builtin_amdgcn_sched_barrier(0);
            KB_SP_MFMA8(0, 2, fq0);
            fq1.lo = read_b8(stageB, 3, 0);
            fq1.hi = read_b8(stageB, 3, 1);
            __builtin_amdgcn_sched_barrier(0);
            KB_SP_MFMA8(1, 2, fq0);
            KB_SP_LOAD(2);
            KB_SP_MFMA8(0, 3, fq1);
            fq0.lo = read_b8(xB, 0, 0);
            fq0.hi = read_b8(xB, 0, 1);
            __builtin_amdgcn_sched_barrier(0);
            KB_SP_LOAD(3);
            KB_SP_MFMA8(1, 3, fq1);
#undef KB_SP_MFMA8
            __builtin_amdgcn_s_setprio(0);
            if constexpr (C::IL) finish_iteration_il();
            else finish_iteration(c_now, qb_now);
        };
        for (int g = 0; g < total; g += 2) {
            iteration8(g, fa0, fa1);
            if (g + 1 < total) iteration8(g + 1, fa1, fa0);
        }
    }
#undef KB_SP_MFMA
#undef KB_SP_LOAD

    if (!SAMPLE) flush_records(p, my_region, wave_cnt, blockIdx.x * NW + wave);      // what is left in the region
}

template <class C> hipError_t launch_scan_sp_cfg(bool sample, int grid, const ScanArgs &a, hipStream_t s)
{
    static LdsAllowed allowed[2];
    auto *fn = sample ? &kb_scan_sp_kernel<C, true> : &kb_scan_sp_kernel<C, false>;
    if (hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(fn), allowed[sample], C::SMEM_BYTES); e != hipSuccess) return e;
    hipExtLaunchKernelGGL(fn, dim3(grid), dim3(C::THREADS), C::SMEM_BYTES, s, scan_timing.start, scan_timing.stop, 0, a);
    return hipGetLastError();
}

}  // namespace kbi
