// The large-batch scan kernel, full-line version: 256 key rows x 256 queries per work item on eight wavefronts
// like kb_scan_sp.hpp, but the direct-to-LDS loads fetch 128 bytes of every key row and of every query row at a
// time (gfx950 only; bf16).
//
// Why 128-byte rows.  A direct-to-LDS load instruction moves 1 KiB; with 64-byte row pieces it covers half of
// 16 cache lines and the other halves are asked for again one d-chunk later, with 128-byte pieces it covers 8
// whole lines once.  Measured with the load pattern and the MFMA count of this kernel and nothing else (256
// workgroups, 2^20 x 1024 bf16 keys, 256 queries): 64-byte pieces 0.47 ms, 128-byte pieces for the keys only
// 0.44 ms, for both operands 0.36 ms, which is what streaming the keys alone takes.
//
// The price is LDS: a d-chunk is now 64 elements, 32 KiB of keys + 32 KiB of queries, and a key piece issued
// now lands about two chunk times later (HBM under load).  So the chunk is worked through in two PHASES, one
// per PIECE of keys (16 KiB: 128 rows x 128 bytes), and the ring is kept in pieces: with 256-query blocks five
// of keys (one in use, four in flight) and four of queries (one chunk in use, the next one landing).  In phase
// f = 2 g + rh a wave (wm, wn) multiplies rows 128 rh + 64 wm + [0, 64) of the tile with queries 64 wn + [0, 64):
// sixteen MFMAs in four k-steps.  Key fragments live in two register sets X and Y (while the MFMAs of one
// k-step run on one set, the other is refilled); the query fragments of all four k-steps are read in the
// chunk's first phase and stay in registers for its second.  One barrier per phase:
//
//   k-step 0 on X, Y <- (f,1);  k-step 1 on Y, X <- (f,2);  k-step 2 on X, Y <- (f,3);
//   wait for my own loads of key piece f+1 (and, rh = 1, of query chunk g+1) and for my LDS reads; BARRIER f
//   (publishes those, retires key piece f and, rh = 0, query chunk g: its fragments are all in registers);
//   k-step 3 on Y, X <- (f+1,0).
//
// Waves 0-3 load keys: piece f+5 (f + the ring depth) into the slot of piece f, from barrier f on.  Waves 4-7
// load queries: chunk g+2 into the slots of chunk g, from barrier 2g on.  Every wave issues exactly ONE load per
// k-step (a steady stream for the texture-address unit instead of bursts after the barriers), nothing about a
// load is decided at run time (past the end of its stream a wave loads its last piece again into slots nobody
// reads), and the loop exists once per kind of wave.  The two kinds keep separate load counters, so the wait for
// a query chunk does not drain the key pieces issued up to four phases ago.
//
// With 128-query blocks (the second configuration) a query chunk is one piece, the ring holds seven key pieces and
// two query pieces (six phases for a key piece to land), and a wave multiplies its 64 rows with 32 queries.
//
// Accumulation order over d, lane-to-element mapping and epilogue are those of the other scan kernels, so the
// scores are bit-identical to theirs.
#pragma once
#include "kb_scan.hpp"

namespace kbi {

// A wave-uniform address pinned to scalar registers at this point of the program: a load from it plus a 32-bit lane
// offset then needs no 64-bit vector arithmetic (and the compiler cannot fold the lane offset into a per-lane pointer
// that it keeps alive across the whole kernel).
__device__ inline const unsigned char *uniform_address(const void *ptr)
{
    const uint64_t v = reinterpret_cast<uint64_t>(ptr);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return reinterpret_cast<const unsigned char *>(((uint64_t)hi << 32) | lo);
}

template <int KT_, int TQ_, bool QF8_ = false> struct WideCfg {
    static constexpr int KT = KT_;
    static constexpr bool QF8 = QF8_;                                // fp8 keys AND fp8 queries: the fp8 matrix instruction
    static constexpr int TK = 256, TQ = TQ_, THREADS = 512, NW = 8;
    static constexpr int KEY_BYTES = KeyTraits<KT>::KEY_BYTES, QRY_BYTES = QF8 ? 1 : KeyTraits<KT>::QRY_BYTES;
    static constexpr int RB = 128;                                   // bytes of a key / query row per d-chunk
    static constexpr int PIECE_ROWS = 128, PIECE_BYTES = PIECE_ROWS * RB;
    static constexpr int NB = TQ / PIECE_ROWS;                       // pieces of a query chunk
    static constexpr int NPB = 2 * NB, NPA = 9 - NPB;                // ring depth in pieces: queries (two chunks), keys (the rest)
    static constexpr int IB = 2, JB = TQ / 128;                      // 32-row blocks of a wave in one phase: keys, queries
    static constexpr int OFF_B = NPA * PIECE_BYTES;
    static constexpr int OFF_AUX = OFF_B + NPB * PIECE_BYTES;
    // side data of a key tile, two copies (item parity)
    static constexpr int AUX_INVK = 0;                       // float  [TK]
    static constexpr int AUX_TAG = AUX_INVK + TK * 4;        // uint64 [TK]
    static constexpr int AUX_LGAIN = AUX_TAG + TK * 8;       // float  [TK]  (weighted random selection only)
    static constexpr int AUX_BYTES = AUX_LGAIN + TK * 4;
    // side data of a query block, one copy
    static constexpr int QAUX_THRP = 0;                      // float  [TQ]
    static constexpr int QAUX_INVQ = QAUX_THRP + TQ * 4;     // float  [TQ]
    static constexpr int QAUX_THR64 = QAUX_INVQ + TQ * 4;    // uint64 [TQ]
    static constexpr int QAUX_QMASK = QAUX_THR64 + TQ * 8;   // uint64 [TQ]
    static constexpr int QAUX_BYTES = QAUX_QMASK + TQ * 8;
    static constexpr int OFF_QAUX = OFF_AUX + 2 * AUX_BYTES;
    static constexpr int SMEM_BYTES = OFF_QAUX + QAUX_BYTES;
    static constexpr int GROUPS_PER_TILE = 8;                // sampling groups: 2 pieces x 2 wave rows x 2 lane halves
    static constexpr int MIN_ROW_BYTES = 4 * RB;             // the key stream runs five pieces ahead of the MFMAs
    static constexpr int KS = QF8 ? 2 : 4;                           // k-steps per chunk: 32 bytes per lane and MFMA for fp8, 16 for bf16
    static_assert(((KT == KB_BF16 && !QF8) || (KT == KB_FP8_E4M3 && QF8 && TQ == 256)) && KEY_BYTES == QRY_BYTES,
                  "written for bf16 keys and queries, and for fp8 keys with fp8 queries in 256-query blocks");
    static_assert(TQ == 256 || TQ == 128, "query blocks of 256 or 128");
    static_assert(NPA % 2 == 1, "the parity of the piece a phase issues is fixed in the code");
    static_assert(SMEM_BYTES <= 160 * 1024, "LDS budget");
};

template <class C, bool SAMPLE, bool DRAW = false>
__global__ __launch_bounds__(512, 1) void kb_scan_wide_kernel(ScanArgs p)
{
    static_assert(!DRAW || (!SAMPLE && !C::QF8), "keys of the weighted random selection: main pass, bf16");
    constexpr int TK = C::TK, TQ = C::TQ, RB = C::RB, IB = C::IB, JB = C::JB, NW = C::NW, PB = C::PIECE_BYTES;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    // LDS addresses are kept as 32-bit pointers of the LDS address space: arithmetic on them is one scalar add, where a
    // generic pointer costs a conversion (with its null check) at every load
    typedef __attribute__((address_space(3))) unsigned char lds_u8;
    typedef __attribute__((address_space(3))) void *lds_ptr;
    typedef const __attribute__((address_space(3))) u32x4 lds_u32x4;
    lds_u8 *const lds = (lds_u8 *)smem;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave & 1, wn = wave >> 1;
    const int lrow = lane & 31, half = lane >> 5;
    const bool filter = p.qmask != nullptr;

    const int nqb = p.nqb;
    const int64_t n_items = p.n_tiles * nqb;
    const int vb = item_lane(blockIdx.x, gridDim.x, nqb);      // this workgroup takes items vb, vb + gridDim.x, ...
    // A sampling pass is launched with one workgroup per item: nothing of the item loop stays live in its epilogue,
    // which looks at every element and needs the registers (a spilled register costs this kernel dearly: its
    // reload queues behind the stream loads in flight).
    const int my_items = SAMPLE ? ((int64_t)vb < n_items ? 1 : 0) : ((int64_t)vb < n_items ? (int)((n_items - vb + gridDim.x - 1) / gridDim.x) : 0);
    const int NC = p.d * C::KEY_BYTES / RB;                    // chunks per item
    const int total = my_items * NC;                           // chunks of this workgroup
    const int phases = 2 * total;
    const uint32_t key_row_bytes = (uint32_t)p.d * C::KEY_BYTES, qry_row_bytes = (uint32_t)p.d * C::QRY_BYTES;
    const int step_tile = gridDim.x / nqb, step_qb = gridDim.x % nqb;

    Record *my_region = p.regions + ((size_t)blockIdx.x * NW + wave) * p.region_cap;
    uint32_t wave_cnt = 0;

    // ---- the load streams -------------------------------------------------------------------------------
    // A piece is 16 load instructions of 1 KiB (8 rows x 128 bytes); loading wave ridx issues instructions ridx,
    // ridx+4, ridx+8, ridx+12 of a piece.  The lane that fills physical 16-byte slot s of row r fetches logical
    // slot s ^ swizzle<8>(r); the rows of a wave's four instructions are 32 apart, so they share the swizzle.
    const int role = wave >> 2, ridx = wave & 3;                       // role 0: keys, role 1: queries
    const int ld_row = ridx * 8 + (lane >> 3);                         // row within the piece, instruction 0
    const uint32_t ld_slot = (uint32_t)(((lane & 7) ^ swizzle<8>(ld_row)) * 16);
    // the stream cursor: (tile, query block, chunk) of the next key piece (role 0) / query chunk (role 1) to issue,
    // the address of that chunk in row 0 of the tile / of the query block 0, and the ring slot it goes to
    int ld_tile = vb / nqb, ld_qb = vb % nqb, ld_c = 0, ld_par = 0;
    const unsigned char *ld_src = nullptr;
    lds_u8 *const ld_ring0 = lds + (role == 0 ? 0 : C::OFF_B) + ridx * 1024;
    lds_u8 *ld_dst = ld_ring0;
    int ld_ring = 0;
    // [piece of the chunk][instruction]: bytes from the tile's (the query block's) first row; a sampling pass gathers
    // key rows from anywhere and counts in units of 16 bytes from the first key (the host scatters the sample only
    // when that fits 32 bits)
    constexpr int OSH = SAMPLE ? 4 : 0;
    uint32_t off[2][4];
    auto ld_setup = [&]() {
        int last, base;
        if (role == 0) {
            const int64_t tile_row0 = (int64_t)ld_tile * (SAMPLE ? p.tile_stride : 1) * TK;      // (unless the sample is scattered)
            const int64_t left = p.n_keys - tile_row0;
            last = left < TK ? (int)left - 1 : TK - 1;
            base = 0;
            ld_src = static_cast<const unsigned char *>(p.keys) + ((SAMPLE && p.row_mul) ? 0 : (size_t)tile_row0 * key_row_bytes);
        } else {
            last = p.Q - 1 - ld_qb * TQ;
            base = ld_qb * TQ;
            ld_src = static_cast<const unsigned char *>(p.queries);
        }
        const uint32_t rb = role == 0 ? key_row_bytes : qry_row_bytes;
        const int64_t tile_run = (SAMPLE && role == 0) ? sample_tile_run(p, ld_tile, TK) : 0;
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int r = h * C::PIECE_ROWS + ld_row + j * 32;
                if (SAMPLE && role == 0 && p.row_mul) off[h][j] = (uint32_t)(((uint64_t)sample_row(p, tile_run, ld_tile, TK, r) * rb + ld_slot) >> 4);
                else off[h][j] = ((uint32_t)(base + (r < last ? r : last)) * rb + ld_slot) >> (role == 0 ? OSH : 0);
            }
    };
    // side data of the key tile the key stream is at: 4-byte loads with clamped rows from the caller's arrays
    // (addresses as a wave-uniform base plus a 32-bit lane offset, the form that needs no 64-bit vector arithmetic)
    auto issue_tile_aux = [&]() {       // role 0 only
        lds_u8 *aux = lds + C::OFF_AUX + ld_par * C::AUX_BYTES;
        // the lane's row numbers are formed here each time (two shifts): kept in registers across the chunks they
        // get spilled, and their reload waits for every stream load in flight
        int lane = threadIdx.x & 63;
        asm volatile("" : "+v"(lane));
        if constexpr (SAMPLE) {
            const int64_t tile_run = sample_tile_run(p, ld_tile, TK);
            const int64_t r = sample_row(p, tile_run, ld_tile, TK, ridx * 64 + lane);
            __builtin_amdgcn_global_load_lds((const void *)(p.inv_norm + r), (lds_ptr)(aux + C::AUX_INVK + ridx * 256), 4, 0, 0);
            if (filter) {
#pragma unroll
                for (int h2 = 0; h2 < 2; ++h2) {
                    const int i = ridx * 2 + h2;
                    const int64_t rt = sample_row(p, tile_run, ld_tile, TK, i * 32 + (lane >> 1));
                    __builtin_amdgcn_global_load_lds((const void *)(reinterpret_cast<const uint32_t *>(p.tags + rt) + (lane & 1)),
                                                     (lds_ptr)(aux + C::AUX_TAG + i * 256), 4, 0, 0);
                }
            }
            return;
        }
        const int64_t row0 = (int64_t)ld_tile * TK;
        const int64_t left = p.n_keys - row0;
        const uint32_t last = left < TK ? (uint32_t)left - 1 : TK - 1;
        {
            const uint32_t r = (uint32_t)(ridx * 64 + lane);
            const unsigned char *g = uniform_address(p.inv_norm + row0);
            __builtin_amdgcn_global_load_lds((const void *)(g + (r < last ? r : last) * 4u), (lds_ptr)(aux + C::AUX_INVK + ridx * 256), 4, 0, 0);
        }
        if constexpr (DRAW) {
            const uint32_t r = (uint32_t)(ridx * 64 + lane);
            const unsigned char *g = uniform_address(p.draw.log_gain + row0);
            __builtin_amdgcn_global_load_lds((const void *)(g + (r < last ? r : last) * 4u), (lds_ptr)(aux + C::AUX_LGAIN + ridx * 256), 4, 0, 0);
        }
        if (filter) {
            const unsigned char *g = uniform_address(p.tags + row0);
#pragma unroll
            for (int h2 = 0; h2 < 2; ++h2) {        // tags as dwords: instruction i covers rows [32 i, 32 i + 32)
                const int i = ridx * 2 + h2;
                const uint32_t r = (uint32_t)(i * 32 + (lane >> 1));
                __builtin_amdgcn_global_load_lds((const void *)(g + ((r < last ? r : last) * 8u + (lane & 1) * 4u)),
                                                 (lds_ptr)(aux + C::AUX_TAG + i * 256), 4, 0, 0);
            }
        }
    };
    // side data of a query block: 16-byte loads from the library's padded per-query arrays.  A sampling pass runs
    // before those exist and needs the mask words only: it takes them from the caller's array as dwords with
    // clamped query numbers (instruction i covers queries [32 i, 32 i + 32), two instructions per loading wave
    // and 128 queries).
    auto issue_query_aux = [&](int qb) {    // role 1 only
        lds_u8 *aux = lds + C::OFF_QAUX;
        int lane = threadIdx.x & 63;            // (formed here each time, as in issue_tile_aux)
        asm volatile("" : "+v"(lane));
        const int q0 = qb * TQ;
        if constexpr (SAMPLE) {
            if (filter) {
                const uint32_t last = (uint32_t)(p.Q - 1 - q0);
                const unsigned char *g = uniform_address(p.qmask + q0);
#pragma unroll
                for (int h2 = 0; h2 < TQ / 128; ++h2) {
                    const int i = ridx * (TQ / 128) + h2;
                    const uint32_t r = (uint32_t)(i * 32 + (lane >> 1));
                    __builtin_amdgcn_global_load_lds((const void *)(g + ((r < last ? r : last) * 8u + (lane & 1) * 4u)),
                                                     (lds_ptr)(aux + C::QAUX_QMASK + i * 256), 4, 0, 0);
                }
            }
            return;
        }
        const uint32_t l16 = (uint32_t)lane * 16u;
        if (ridx == 0) {
            if (lane < TQ / 4) {        // TQ floats
                __builtin_amdgcn_global_load_lds((const void *)(uniform_address(p.invq + q0) + l16), (lds_ptr)(aux + C::QAUX_INVQ), 16, 0, 0);
                __builtin_amdgcn_global_load_lds((const void *)(uniform_address(p.thrp + q0) + l16), (lds_ptr)(aux + C::QAUX_THRP), 16, 0, 0);
            }
        } else if (ridx == 1) {
            __builtin_amdgcn_global_load_lds((const void *)(uniform_address(p.thr64 + q0) + l16), (lds_ptr)(aux + C::QAUX_THR64), 16, 0, 0);
            if (TQ == 256)
                __builtin_amdgcn_global_load_lds((const void *)(uniform_address(p.thr64 + q0 + 128) + l16), (lds_ptr)(aux + C::QAUX_THR64 + 1024), 16, 0, 0);
        } else if (ridx == 2 && filter) {
            __builtin_amdgcn_global_load_lds((const void *)(uniform_address(p.qmask_pad + q0) + l16), (lds_ptr)(aux + C::QAUX_QMASK), 16, 0, 0);
            if (TQ == 256)
                __builtin_amdgcn_global_load_lds((const void *)(uniform_address(p.qmask_pad + q0 + 128) + l16), (lds_ptr)(aux + C::QAUX_QMASK + 1024), 16, 0, 0);
        }
    };
    // role 0: load j (0..3) of the key piece at the cursor, half h of its chunk; key_next(h) moves the cursor on
    auto key_issue = [&](int h, int j) {
        __builtin_amdgcn_global_load_lds((const void *)(ld_src + ((uint64_t)off[h][j] << OSH)), (lds_ptr)(ld_dst + j * 4096), 16, 0, 0);
    };
    auto item_next = [&]() {
        if constexpr (SAMPLE) return;       // one item per workgroup: the stream ends with it
        ld_c = 0;
        ld_par ^= 1;
        ld_tile += step_tile;
        ld_qb += step_qb;
        if (ld_qb >= nqb) {
            ld_qb -= nqb;
            ++ld_tile;
        }
        if (role == 0 || nqb > 1) ld_setup();
        else ld_src = static_cast<const unsigned char *>(p.queries);
    };
    // more: another piece follows in the stream.  Past its end the cursor stays where it is: the loop goes on issuing
    // loads (of the last piece again) into ring slots that nobody reads any more, so that nothing in it is conditional.
    auto key_next = [&](int h, bool more) {
        ld_ring = ld_ring + 1 == C::NPA ? 0 : ld_ring + 1;
        ld_dst = ld_ring0 + ld_ring * PB;
        if (more && h == 1) {
            ld_src += RB;
            if (++ld_c == NC) item_next();
        }
    };
    // role 1: load j (0..7) of the query chunk at the cursor: piece j / 4, instruction j % 4
    auto qry_issue = [&](int j) {
        if (j >= 4 * C::NB) return;        // a 128-query chunk is one piece
        __builtin_amdgcn_global_load_lds((const void *)(ld_src + off[j / 4][j % 4]), (lds_ptr)(ld_dst + (j / 4) * PB + (j % 4) * 4096), 16, 0, 0);
    };
    auto qry_next = [&](bool more) {
        ld_ring ^= C::NB;
        ld_dst = ld_ring0 + ld_ring * PB;
        if (more) {
            ld_src += RB;
            if (++ld_c == NC) item_next();
        }
    };

    // ---- fragment addresses -------------------------------------------------------------------------------
    // piece-local row = 64 * (wave's half of the piece) + 32 * block + lrow; logical 16-byte slot of k-step kk = 2 kk + half
    // (kk << 5 only touches bits 5 and 6, a ring slot is a multiple of 16 KiB: the XOR can follow the addition)
    constexpr bool F8 = C::QF8;
    const int hslot = F8 ? 2 * half : half;                            // a lane's first 16-byte slot within a k-step
    const int baseA = (wm * 64 + lrow) * RB | ((hslot ^ swizzle<8>(lrow)) << 4);
    const int qrow = wn * (32 * JB) + lrow;                            // this lane's query in block 0 of the wave
    const int baseB = C::OFF_B + (qrow / C::PIECE_ROWS) * PB + ((qrow % C::PIECE_ROWS) * RB | ((hslot ^ swizzle<8>(lrow)) << 4));
    // bf16: 16 bytes of the row per lane and k-step (slot 2 kk + half); fp8: 32 bytes (slots 4 kk + 2 half, + 1)
    typedef int i32x8 __attribute__((ext_vector_type(8)));
    typedef int i32x4 __attribute__((ext_vector_type(4)));
    typedef typename std::conditional<F8, i32x8, u32x4>::type Frag;
    auto read_f = [&](int addr, int kk, int blk) {
        if constexpr (F8) {
            i32x8 v;
            v.lo = __builtin_bit_cast(i32x4, *(lds_u32x4 *)(lds + ((addr ^ (kk << 6)) + blk * 32 * RB)));
            v.hi = __builtin_bit_cast(i32x4, *(lds_u32x4 *)(lds + (((addr ^ (kk << 6)) ^ 16) + blk * 32 * RB)));
            return v;
        } else {
            return *(lds_u32x4 *)(lds + ((addr ^ (kk << 5)) + blk * 32 * RB));
        }
    };

    f32x16 acc[2][IB][JB];      // (never cleared: every item's first MFMAs start from zero)

    auto epilogue = [&](int tile, int qb, int par, int qrow, int half) {
        const unsigned char *aux = smem + C::OFF_AUX + par * C::AUX_BYTES, *qaux = smem + C::OFF_QAUX;
        const EpiSide sd{reinterpret_cast<const float *>(aux + C::AUX_INVK), reinterpret_cast<const uint64_t *>(aux + C::AUX_TAG),
                         reinterpret_cast<const float *>(qaux + C::QAUX_THRP), reinterpret_cast<const float *>(qaux + C::QAUX_INVQ),
                         reinterpret_cast<const uint64_t *>(qaux + C::QAUX_THR64), reinterpret_cast<const uint64_t *>(qaux + C::QAUX_QMASK),
                         reinterpret_cast<const float *>(aux + C::AUX_LGAIN)};
        const int64_t row0 = SAMPLE ? sample_row0(p, tile, TK) : (int64_t)tile * TK;
        const int64_t tile_run = SAMPLE ? sample_tile_run(p, tile, TK) : 0;
#pragma unroll
        for (int rh = 0; rh < 2; ++rh) {
            if constexpr (SAMPLE)       // sampling groups: (piece, wave row, lane half) = 32 rows each
                sample_epilogue<IB, JB>(acc[rh], sd, filter, rh * 128 + wm * 64, qrow, half, row0, qb * TQ, p,
                                        (int64_t)tile * C::GROUPS_PER_TILE + (rh * 2 + wm) * 2 + half, tile_run, TK);
            else if constexpr (DRAW)
                main_epilogue_draw<IB, JB>(acc[rh], sd, filter, rh * 128 + wm * 64, qrow, half, row0, qb * TQ, p, my_region, wave_cnt, blockIdx.x * NW + wave);
            else
                main_epilogue<IB, JB, F8>(acc[rh], sd, filter, rh * 128 + wm * 64, qrow, half, row0, qb * TQ, p, my_region, wave_cnt, blockIdx.x * NW + wave);
        }
    };

    if (total > 0) {        // uniform over the workgroup
        // ---- prologue ---------------------------------------------------------------------------------------------
        // keys: all pieces of the ring but the last, and the first instruction of that one (every item has at least
        // four chunks = eight pieces); queries: chunk 0 and the first five instructions of chunk 1.  From here on every
        // wave issues one load per k-step.
        ld_setup();
        if (role == 0) {
            issue_tile_aux();
#pragma unroll
            for (int s = 0; s < C::NPA - 1; ++s) {
#pragma unroll
                for (int j = 0; j < 4; ++j) key_issue(s & 1, j);
                key_next(s & 1, true);
            }
            key_issue(0, 0);
            if (F8) key_issue(0, 1);                                   // (two loads per k-step there: two k-steps per phase)
            __builtin_amdgcn_s_waitcnt(waitcnt_vm(4 * (C::NPA - 2) + (F8 ? 2 : 1)));   // piece 0 (and the side data before it) has landed
        } else {
            issue_query_aux(vb % nqb);
#pragma unroll
            for (int j = 0; j < 8; ++j) qry_issue(j);
            qry_next(true);
#pragma unroll
            for (int j = 0; j < (F8 ? 6 : 5); ++j) qry_issue(j);
            __builtin_amdgcn_s_waitcnt(waitcnt_vm(F8 ? 6 : C::NB == 2 ? 5 : 4));     // chunk 0 (and the side data before it) has landed
        }
        __builtin_amdgcn_s_waitcnt(waitcnt_lgkm0());
        bare_barrier();

        int tile = vb / nqb, qb = vb % nqb, par = 0;
        int ra = 0, rb = 0;                                    // ring slots: key piece of the phase, first query piece of the chunk
        int f = 0;                                             // phase index
        // key fragments of one k-step in two sets (one in use, one being refilled); the query fragments of all four
        // k-steps of the chunk stay in registers for its second phase
        Frag xa[IB], ya[IB], fb[C::KS][JB];
#pragma unroll
        for (int ib = 0; ib < IB; ++ib) xa[ib] = read_f(baseA, 0, ib);
#pragma unroll
        for (int jb = 0; jb < JB; ++jb) fb[0][jb] = read_f(baseB, 0, jb);

        // (KU: the k-step.  In an item's first chunk, the MFMAs of k-step 0 start from the constant zero instead of the
        // accumulator: nothing has to clear 128 registers between two items)
#define KBW_MFMA(RH, SA, KU, I, J)                                                                                                  \
    if constexpr (F8)                                                                                                               \
        acc[RH][I][J] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(SA[I], fb[KU][J], (FIRST && KU == 0) ? zero16 : acc[RH][I][J], 0, 0, 0, 0, 0, 0); \
    else                                                                                                                            \
        acc[RH][I][J] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, SA[I]), __builtin_bit_cast(bf16x8, fb[KU][J]), \
                                                                (FIRST && KU == 0) ? zero16 : acc[RH][I][J], 0, 0, 0);             \
    __builtin_amdgcn_sched_barrier(0)
        // one k-step: four MFMAs (two with 128-query blocks) on the key fragments SA and the query fragments fb[KU]; meanwhile the key fragments DA
        // are refilled from the piece at AA, k-step KR, and (KBW_KSTEP_AB) the query fragments fb[KR] from the chunk at
        // AB; L0 .. L3: what this wave loads after each of the MFMAs
#define KBW_KSTEP_AB(RH, SA, KU, DA, AA, AB, KR, L0, L1, L2, L3) \
    KBW_MFMA(RH, SA, KU, 0, 0);                              \
    DA[0] = read_f(AA, KR, 0);                                   \
    fb[KR][0] = read_f(AB, KR, 0);                               \
    L0;                                                          \
    __builtin_amdgcn_sched_barrier(0);                           \
    if constexpr (JB == 2) {                                     \
        KBW_MFMA(RH, SA, KU, 0, 1);                          \
        fb[KR][1] = read_f(AB, KR, 1);                           \
    }                                                            \
    DA[1] = read_f(AA, KR, 1);                                   \
    L1;                                                          \
    __builtin_amdgcn_sched_barrier(0);                           \
    KBW_MFMA(RH, SA, KU, 1, 0);                              \
    L2;                                                          \
    __builtin_amdgcn_sched_barrier(0);                           \
    if constexpr (JB == 2) {                                     \
        KBW_MFMA(RH, SA, KU, 1, 1);                          \
    }                                                            \
    L3;                                                          \
    __builtin_amdgcn_sched_barrier(0)
#define KBW_KSTEP_A(RH, SA, KU, DA, AA, KR, L0, L1, L2, L3) \
    KBW_MFMA(RH, SA, KU, 0, 0);                         \
    DA[0] = read_f(AA, KR, 0);                              \
    L0;                                                     \
    __builtin_amdgcn_sched_barrier(0);                      \
    if constexpr (JB == 2) {                                \
        KBW_MFMA(RH, SA, KU, 0, 1);                     \
    }                                                       \
    DA[1] = read_f(AA, KR, 1);                              \
    L1;                                                     \
    __builtin_amdgcn_sched_barrier(0);                      \
    KBW_MFMA(RH, SA, KU, 1, 0);                         \
    L2;                                                     \
    __builtin_amdgcn_sched_barrier(0);                      \
    if constexpr (JB == 2) {                                \
        KBW_MFMA(RH, SA, KU, 1, 1);                     \
    }                                                       \
    L3;                                                     \
    __builtin_amdgcn_sched_barrier(0)
        // fp8: the MFMAs are twice as long and the fragments twice as wide, so the key fragments have ONE register set:
        // block ib is refilled (piece at AA, k-step KR) right after its two MFMAs, two MFMAs before it is used again;
        // two loads per k-step (L0, L1), since a phase has two k-steps
#define KBW_KSTEP8(RH, KU, AA, KR, RB0, RB1, L0, L1) \
    KBW_MFMA(RH, xa, KU, 0, 0);                  \
    RB0;                                             \
    L0;                                              \
    __builtin_amdgcn_sched_barrier(0);               \
    KBW_MFMA(RH, xa, KU, 0, 1);                  \
    xa[0] = read_f(AA, KR, 0);                       \
    RB1;                                             \
    __builtin_amdgcn_sched_barrier(0);               \
    KBW_MFMA(RH, xa, KU, 1, 0);                  \
    L1;                                              \
    __builtin_amdgcn_sched_barrier(0);               \
    KBW_MFMA(RH, xa, KU, 1, 1);                  \
    xa[1] = read_f(AA, KR, 1);                       \
    __builtin_amdgcn_sched_barrier(0)
#define KBW_NONE (void)0

        // The chunks of one item, for a wave of kind ROLE (the two kinds differ only in what they load and wait for,
        // and each gets its own copy of the loop so that none of it is decided per load).
        // Wait before barrier f.  Key waves: piece f+1 has landed once at most the pieces f+2 .. f+4 are outstanding.
        // Query waves: chunk g+1 is needed from barrier 2g+1 on; they issued nothing since the first half of the phase
        // before, so they wait for everything.
        auto item_chunks = [&](auto role_c, int g0) {
            constexpr int ROLE = decltype(role_c)::value;
            auto wait_before_barrier = [&](int rh) {
                if (ROLE == 0) __builtin_amdgcn_s_waitcnt(waitcnt_vm(4 * (C::NPA - 2)));
                else if (rh == 1) __builtin_amdgcn_s_waitcnt(waitcnt_vm(4));
                __builtin_amdgcn_s_waitcnt(waitcnt_lgkm0());
                __builtin_amdgcn_sched_barrier(0);
                bare_barrier();
                __builtin_amdgcn_sched_barrier(0);
            };
            auto chunk = [&](auto first_c, int c) {
                constexpr bool FIRST = decltype(first_c)::value;
                const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                const int g = g0 + c;
                // ======== phase 2g: key piece in slot ra, query chunk in slots rb, rb+1 ========
                {
                    const int ran = ra + 1 == C::NPA ? 0 : ra + 1;
                    const int aa = baseA + ra * PB, ab = baseB + rb * PB, aan = baseA + ran * PB;
                    // query waves: chunk g+1 into the slots that barrier 2g-1 retired; key waves: piece f+NPA (second half
                    // of chunk g+2) into the slot that barrier f retires
                    __builtin_amdgcn_s_setprio(1);
                    if constexpr (!F8) {
                        KBW_KSTEP_AB(0, xa, 0, ya, aa, ab, 1, KBW_NONE, KBW_NONE, if (ROLE == 0) key_issue(0, 1); else qry_issue(5), KBW_NONE);
                        KBW_KSTEP_AB(0, ya, 1, xa, aa, ab, 2, KBW_NONE, KBW_NONE, if (ROLE == 0) key_issue(0, 2); else qry_issue(6), KBW_NONE);
                        KBW_KSTEP_AB(0, xa, 2, ya, aa, ab, 3, KBW_NONE, KBW_NONE,
                                     if (ROLE == 0) { key_issue(0, 3); key_next(0, true); } else { qry_issue(7); qry_next(g + 2 < total); }, KBW_NONE);
                    } else {        // two k-steps per phase and two loads per k-step; the barrier comes after the first k-step
                        KBW_KSTEP8(0, 0, aa, 1, fb[1][0] = read_f(ab, 1, 0), fb[1][1] = read_f(ab, 1, 1), if (ROLE == 0) key_issue(0, 2); else qry_issue(6),
                                   if (ROLE == 0) { key_issue(0, 3); key_next(0, true); } else { qry_issue(7); qry_next(g + 2 < total); });
                    }
                    __builtin_amdgcn_s_setprio(0);
                    wait_before_barrier(0);
                    // a new query block's side data: every epilogue of the previous item ended before this barrier
                    if (ROLE == 1 && nqb > 1 && c == 0 && g > 0) issue_query_aux(qb);
                    __builtin_amdgcn_s_setprio(1);
                    if constexpr (!F8) {
                        KBW_KSTEP_A(0, ya, 3, xa, aan, 0, KBW_NONE, KBW_NONE, if (ROLE == 0) key_issue(1, 0); else qry_issue(0), KBW_NONE);
                    } else {
                        KBW_KSTEP8(0, 1, aan, 0, KBW_NONE, KBW_NONE, if (ROLE == 0) key_issue(1, 0); else qry_issue(0),
                                   if (ROLE == 0) key_issue(1, 1); else qry_issue(1));
                    }
                    __builtin_amdgcn_s_setprio(0);
                    ra = ran;
                    ++f;
                }
                // ======== phase 2g+1 ========
                {
                    const int ran = ra + 1 == C::NPA ? 0 : ra + 1, rbn = rb ^ C::NB;
                    const bool more = g + 1 < total;
                    const int aa = baseA + ra * PB;
                    // past the last chunk the refill of X reads the current slots again (valid memory, values unused)
                    const int aan = baseA + (more ? ran : ra) * PB, abn = baseB + (more ? rbn : rb) * PB;
                    // key waves: piece f+NPA (the first half of its chunk) and, before it, the side data of a new tile
                    __builtin_amdgcn_s_setprio(1);
                    if constexpr (!F8) {
                        KBW_KSTEP_A(1, xa, 0, ya, aa, 1, KBW_NONE, KBW_NONE, if (ROLE == 0) key_issue(1, 1); else qry_issue(1), KBW_NONE);
                        KBW_KSTEP_A(1, ya, 1, xa, aa, 2, KBW_NONE, KBW_NONE, if (ROLE == 0) key_issue(1, 2); else qry_issue(2), KBW_NONE);
                        KBW_KSTEP_A(1, xa, 2, ya, aa, 3, KBW_NONE, KBW_NONE,
                                    if (ROLE == 0) { key_issue(1, 3); key_next(1, f + C::NPA < phases); } else qry_issue(3), KBW_NONE);
                    } else {
                        KBW_KSTEP8(1, 0, aa, 1, KBW_NONE, KBW_NONE, if (ROLE == 0) key_issue(1, 2); else qry_issue(2),
                                   if (ROLE == 0) { key_issue(1, 3); key_next(1, f + C::NPA < phases); } else qry_issue(3));
                    }
                    __builtin_amdgcn_s_setprio(0);
                    wait_before_barrier(1);
                    if (ROLE == 0 && ld_c == 0 && f + C::NPA < phases) issue_tile_aux();
                    __builtin_amdgcn_s_setprio(1);
                    if constexpr (!F8) {
                        KBW_KSTEP_AB(1, ya, 3, xa, aan, abn, 0, KBW_NONE, KBW_NONE, if (ROLE == 0) key_issue(0, 0); else qry_issue(4), KBW_NONE);
                    } else {
                        KBW_KSTEP8(1, 1, aan, 0, fb[0][0] = read_f(abn, 0, 0), fb[0][1] = read_f(abn, 0, 1), if (ROLE == 0) key_issue(0, 0); else qry_issue(4),
                                   if (ROLE == 0) key_issue(0, 1); else qry_issue(5));
                    }
                    __builtin_amdgcn_s_setprio(0);
                    ra = ran;
                    rb = rbn;
                    ++f;
                }
            };
            chunk(std::true_type{}, 0);
            for (int c = 1; c < NC; ++c) chunk(std::false_type{}, c);
        };

        for (int it = 0; it < my_items; ++it) {
            if (role == 0) item_chunks(std::integral_constant<int, 0>{}, it * NC);
            else item_chunks(std::integral_constant<int, 1>{}, it * NC);
            {
                // What the epilogue derives from the item's coordinates (addresses of its outputs, row numbers) is
                // computed here and not, as the compiler would have it when a workgroup has a single item, before
                // the chunks, where it would sit in registers the contraction needs.
                // The same for what it derives from the lane's place in the tile (LDS addresses of the lane's query
                // and rows): kept across the chunks these cost registers that end up spilled, and a reload
                // queues behind the stream loads in flight.
                int tile_e = tile, qb_e = qb, par_e = par, qrow_e = qrow, half_e = half;
                asm volatile("" : "+s"(tile_e), "+s"(qb_e), "+s"(par_e), "+v"(qrow_e), "+v"(half_e));
                epilogue(tile_e, qb_e, par_e, qrow_e, half_e);
            }
            par ^= 1;
            tile += step_tile;
            qb += step_qb;
            if (qb >= nqb) {
                qb -= nqb;
                ++tile;
            }
        }
#undef KBW_KSTEP_AB
#undef KBW_KSTEP8
#undef KBW_KSTEP_A
#undef KBW_NONE
#undef KBW_MFMA
        __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));             // the loads past the end of the stream
    }

    if (!SAMPLE) flush_records(p, my_region, wave_cnt, blockIdx.x * NW + wave);      // what is left in the region
}

template <class C> hipError_t launch_scan_wide_cfg(bool sample, int grid, const ScanArgs &a, hipStream_t s)
{
    static LdsAllowed allowed[3];
    const bool draw = a.draw.enabled != 0;
    if (C::QF8 && (sample || draw)) return hipErrorInvalidValue;     // fp8: the sampling pass runs the 64-byte-piece kernel (fewer registers)
    if (draw && sample) return hipErrorInvalidValue;                 // keys of the weighted random selection: main pass only
    auto *fn = (sample && !C::QF8) ? &kb_scan_wide_kernel<C, C::QF8 ? false : true>
               : (draw && !C::QF8) ? &kb_scan_wide_kernel<C, false, C::QF8 ? false : true> : &kb_scan_wide_kernel<C, false>;
    if (hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(fn), allowed[draw ? 2 : sample], C::SMEM_BYTES); e != hipSuccess) return e;
    hipExtLaunchKernelGGL(fn, dim3(grid), dim3(C::THREADS), C::SMEM_BYTES, s, scan_timing.start, scan_timing.stop, 0, a);
    return hipGetLastError();
}

}  // namespace kbi
