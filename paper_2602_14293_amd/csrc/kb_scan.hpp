// The scan kernel: similarity contraction on MFMA with the score scaling, tag predicate and
// threshold filter fused into its epilogue (gfx950 only).
//
// Work decomposition.  One work item = (key tile of TK rows) x (query block of TQ queries) x all of d.
// A persistent workgroup walks items v, v + gridDim.x, ... (v = item_lane(blockIdx.x)) with the query block as
// the fastest index, so concurrently running workgroups share a key tile through L2 when Q > TQ.
// The contraction runs as S^T = K * Q^T: key rows are the MFMA "A" operand (M dimension), queries the
// "B" operand (N dimension).  In the 32x32 accumulator layout a lane then owns ONE query column and 16
// key rows per block, so every per-query quantity (threshold, mask word, 1/|q|) is lane-local.
//
// Data movement.  Keys and queries are both row-major with d contiguous, which is exactly the
// k-contiguous fragment layout MFMA wants for A and for B^T, so no transpose exists anywhere.
// Each d-chunk (RBA bytes of every key row, RBB bytes of every query row) goes HBM/L2 -> LDS with
// 16-byte direct-to-LDS loads (no VGPR round trip).  A direct load writes LDS at
// wave-uniform base + lane * 16, so the bank-conflict-avoiding XOR swizzle is applied on the global
// side: the lane that fills physical 16-byte slot pp of row r fetches logical slot pp ^ swz(r).
// NSTAGE chunk buffers are in flight; one barrier per chunk.
//
// Epilogue.  The sampling pass keeps, per lane and query, the best qualifying candidate of the lane's
// rows (one "group") and stores it; the k-th best group maximum is a valid lower bound of the k-th best
// score.  The main pass tests dot * inv_k against a per-query pre-filter with one FMA + max per element,
// and only in blocks in which some lane passes do the passing lanes apply the tag predicate and append
// (raw dot product, row, query) to their wave's private record region (slot = the wave's running count +
// the lane's rank, plain global store); the wave moves its records to the per-query lists itself.
#pragma once
#include <type_traits>
#include "kb_epilogue.hpp"
#include "kb_internal.hpp"

namespace kbi {

template <int KT> struct KeyTraits;
template <> struct KeyTraits<KB_F32> { static constexpr int KEY_BYTES = 4, QRY_BYTES = 4; };
template <> struct KeyTraits<KB_BF16> { static constexpr int KEY_BYTES = 2, QRY_BYTES = 2; };
template <> struct KeyTraits<KB_FP8_E4M3> { static constexpr int KEY_BYTES = 1, QRY_BYTES = 2; };
template <> struct KeyTraits<KB_FP8_Q8> { static constexpr int KEY_BYTES = 1, QRY_BYTES = 1; };

// One k-group = 32 bytes of a key row: lane half h owns bytes [16h, 16h+16) of it.
//   bf16: 16 elements, one 32x32x16 MFMA.          query bytes [16h, +16) of the group's 32
//   f32 :  8 elements, four 32x32x2 MFMAs.         query bytes [16h, +16) of the group's 32
//   fp8 : 32 elements, two 32x32x16 bf16 MFMAs after an exact e4m3 -> bf16 widening;
//         query bytes [32h, +32) of the group's 64 (two 16-byte pieces).
// fp8 keys with fp8 queries: one k-group = 64 bytes of a key row and of a query row, one 32x32x64 fp8 MFMA; lane half
// h owns bytes [32h, 32h+32) of either (two 16-byte pieces), the operand layout of every kernel that takes fp8 queries.
template <int KT> struct Mma;

template <> struct Mma<KB_BF16> {
    typedef u32x4 PrepA;
    static __device__ inline PrepA prepare(u32x4 a) { return a; }
    static __device__ inline void run(f32x16 &acc, const PrepA &a, u32x4 b0, u32x4)
    {
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b0),
                                                      acc, 0, 0, 0);
    }
};

template <> struct Mma<KB_F32> {
    typedef u32x4 PrepA;
    static __device__ inline PrepA prepare(u32x4 a) { return a; }
    static __device__ inline void run(f32x16 &acc, const PrepA &a, u32x4 b0, u32x4)
    {
#pragma unroll
        for (int e = 0; e < 4; ++e)
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(as_f32(a[e]), as_f32(b0[e]), acc, 0, 0, 0);
    }
};

// e4m3 has 3 mantissa bits and a 4-bit exponent, so every code is exactly a bf16 value: one gfx950 conversion
// instruction (v_cvt_scalef32_pk_bf16_fp8, scale 1) turns two codes into a packed pair of bf16 values.
__device__ inline uint32_t e4m3_pair_to_bf16(uint32_t word, bool upper)
{
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    const bf16x2 v = upper ? __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(word, 1.0f, true) : __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(word, 1.0f, false);
    return __builtin_bit_cast(uint32_t, v);
}

template <> struct Mma<KB_FP8_E4M3> {
    struct PrepA {
        u32x4 lo, hi;
    };
    static __device__ inline PrepA prepare(u32x4 a)
    {
        PrepA p;
        p.lo = u32x4{e4m3_pair_to_bf16(a.x, false), e4m3_pair_to_bf16(a.x, true), e4m3_pair_to_bf16(a.y, false),
                     e4m3_pair_to_bf16(a.y, true)};
        p.hi = u32x4{e4m3_pair_to_bf16(a.z, false), e4m3_pair_to_bf16(a.z, true), e4m3_pair_to_bf16(a.w, false),
                     e4m3_pair_to_bf16(a.w, true)};
        return p;
    }
    static __device__ inline void run(f32x16 &acc, const PrepA &a, u32x4 b0, u32x4 b1)
    {
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a.lo), __builtin_bit_cast(bf16x8, b0),
                                                      acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a.hi), __builtin_bit_cast(bf16x8, b1),
                                                      acc, 0, 0, 0);
    }
};

template <> struct Mma<KB_FP8_Q8> {
    struct PrepA {
        u32x4 lo, hi;
    };
    static __device__ inline void run(f32x16 &acc, const PrepA &a, u32x4 b0, u32x4 b1)
    {
        typedef int i32x8 __attribute__((ext_vector_type(8)));
        const i32x8 av = {(int)a.lo[0], (int)a.lo[1], (int)a.lo[2], (int)a.lo[3], (int)a.hi[0], (int)a.hi[1], (int)a.hi[2], (int)a.hi[3]};
        const i32x8 bv = {(int)b0[0], (int)b0[1], (int)b0[2], (int)b0[3], (int)b1[0], (int)b1[1], (int)b1[2], (int)b1[3]};
        acc = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(av, bv, acc, 0, 0, 0, 0, 0, 0);
    }
};

// XOR swizzle of the 16-byte slots of a row with PPR slots: 16 consecutive rows at one logical slot
// touch 16 different slots modulo 256 bytes, i.e. all 64 LDS banks once.
template <int PPR> __device__ inline int swizzle(int row)
{
    static_assert(PPR == 4 || PPR == 8 || PPR == 16, "row bytes must be 64, 128 or 256");
    return PPR == 4 ? (row >> 2) & 3 : PPR == 8 ? (row >> 1) & 7 : row & 15;
}

constexpr int waitcnt_vm(int n) { return (n & 15) | ((n >> 4) << 14) | 0x0070 | 0x0F00; }

template <int KT_, int TK_, int TQ_, int WM_, int WN_, int RBA_, int NSTAGE_, int WGPC_>
struct ScanCfg {
    static constexpr int KT = KT_, TK = TK_, TQ = TQ_, WM = WM_, WN = WN_, RBA = RBA_, NSTAGE = NSTAGE_, WGPC = WGPC_;
    static constexpr int KEY_BYTES = KeyTraits<KT>::KEY_BYTES, QRY_BYTES = KeyTraits<KT>::QRY_BYTES;
    static constexpr int BMUL = QRY_BYTES / KEY_BYTES;
    static constexpr int RBB = RBA * BMUL;
    static constexpr int PPRA = RBA / 16, PPRB = RBB / 16;
    static constexpr bool Q8 = KT == KB_FP8_Q8;
    static constexpr int KG = RBA / (Q8 ? 64 : 32);
    static constexpr int NW = WM * WN, THREADS = 64 * NW;
    static constexpr int IB = TK / WM / 32, JB = TQ / WN / 32;
    static constexpr int A_BYTES = TK * RBA, B_BYTES = TQ * RBB, STAGE_BYTES = A_BYTES + B_BYTES;
    static constexpr int NIA = A_BYTES / 1024, NIB = B_BYTES / 1024;   // wave-wide load instructions per chunk
    static constexpr int VM_PER_CHUNK = NIA / NW + NIB / NW;           // fewest loads any wave issues per chunk
    static constexpr int OFF_INVK = NSTAGE * STAGE_BYTES;
    static constexpr int OFF_TAG = OFF_INVK + TK * 4;
    static constexpr int OFF_THR64 = OFF_TAG + TK * 8;
    static constexpr int OFF_QMASK = OFF_THR64 + TQ * 8;
    static constexpr int OFF_INVQ = OFF_QMASK + TQ * 8;
    static constexpr int OFF_THRP = OFF_INVQ + TQ * 4;
    static constexpr int OFF_LGAIN = OFF_THRP + TQ * 4;
    static constexpr int SMEM_BYTES = OFF_LGAIN + TK * 4;
    static constexpr int GROUPS_PER_TILE = WM * 2;
    static_assert(TK % (WM * 32) == 0 && TQ % (WN * 32) == 0, "wave tiles are made of 32x32 blocks");
    static_assert(A_BYTES % 1024 == 0 && B_BYTES % 1024 == 0, "chunk buffers are filled 1 KiB per wave instruction");
    static_assert(THREADS >= TK && THREADS >= TQ, "one thread stages one row's side data");
    static_assert(SMEM_BYTES * WGPC <= 160 * 1024, "LDS budget");
    static_assert(VM_PER_CHUNK * (NSTAGE - 2) < 64, "vmcnt is a 6-bit counter");
};

constexpr int waitcnt_lgkm0() { return 0xC07F; }   // lgkmcnt(0), nothing else

// Workgroups are dealt to the eight XCDs round-robin by block index, and each XCD has an L2 of its own.  When a
// key tile is scored against several query blocks (items that differ in the query block only are consecutive),
// the workgroups of one XCD take consecutive items, so that a tile's re-reads meet in one L2.
__device__ inline int item_lane(int block, int grid, int nqb)
{
    constexpr int XCDS = 8;
    if (nqb == 1 || grid % XCDS != 0) return block;
    return (block % XCDS) * (grid / XCDS) + block / XCDS;
}


// Workgroup barrier without the fence semantics of __syncthreads(): the fence would drain every
// outstanding direct-to-LDS load (vmcnt(0)) and with it the prefetch pipeline.  Callers wait for exactly
// the counters they need first.
__device__ inline void bare_barrier()
{
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

template <class C, bool SAMPLE, bool DRAW>
__global__ __launch_bounds__(C::THREADS, C::WGPC) void kb_scan_kernel(ScanArgs p)
{
    constexpr int TK = C::TK, TQ = C::TQ, RBA = C::RBA, RBB = C::RBB, IB = C::IB, JB = C::JB, NW = C::NW;
    constexpr int LA = C::NIA / NW, LB = C::NIB / NW;           // load instructions per wave per chunk
    constexpr int RSTEP_A = NW * 64 / C::PPRA, RSTEP_B = NW * 64 / C::PPRB;   // rows between a wave's instructions
    static_assert(C::NIA % NW == 0 && C::NIB % NW == 0, "every wave issues the same number of loads");
    static_assert(RSTEP_A % 32 == 0 && RSTEP_B % 32 == 0, "the swizzle must not change between instructions");
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    typedef __attribute__((address_space(3))) void *lds_ptr;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / C::WN, wn = wave % C::WN;
    const int lrow = lane & 31, half = lane >> 5;
    const bool filter = p.qmask != nullptr;

    float *aux_invk = reinterpret_cast<float *>(smem + C::OFF_INVK);
    uint64_t *aux_tag = reinterpret_cast<uint64_t *>(smem + C::OFF_TAG);
    uint64_t *aux_thr64 = reinterpret_cast<uint64_t *>(smem + C::OFF_THR64);
    uint64_t *aux_qmask = reinterpret_cast<uint64_t *>(smem + C::OFF_QMASK);
    float *aux_invq = reinterpret_cast<float *>(smem + C::OFF_INVQ);
    float *aux_lgain = reinterpret_cast<float *>(smem + C::OFF_LGAIN);

    // items: (tile, qb) with qb fastest
    const int nqb = p.nqb;
    const int64_t tstride = p.tile_stride;     // 1, or the distance between the tiles of a sampling pass
    const int64_t n_items = p.n_tiles * nqb;
    const int vb = item_lane(blockIdx.x, gridDim.x, nqb);      // this workgroup takes items vb, vb + gridDim.x, ...
    const int my_items = (int64_t)vb < n_items ? (int)((n_items - vb + gridDim.x - 1) / gridDim.x) : 0;
    const int NC = p.d * C::KEY_BYTES / RBA;          // chunks per row
    const int total = my_items * NC;
    const uint32_t key_row_bytes = (uint32_t)p.d * C::KEY_BYTES, qry_row_bytes = (uint32_t)p.d * C::QRY_BYTES;
    const int step_tile = gridDim.x / nqb, step_qb = gridDim.x % nqb;

    Record *my_region = p.regions + ((size_t)blockIdx.x * NW + wave) * p.region_cap;
    uint32_t wave_cnt = 0;       // wave-uniform

    // ---- the load stream: chunk after chunk, item after item ------------------------------------
    // lane -> (row, 16-byte slot) of the 1 KiB block a wave instruction fills; same slot for all of them
    const int ldA_row = (wave * 64 + lane) / C::PPRA, ldB_row = (wave * 64 + lane) / C::PPRB;
    const uint32_t ldA_piece = (uint32_t)((((wave * 64 + lane) % C::PPRA) ^ swizzle<C::PPRA>(ldA_row)) * 16);
    const uint32_t ldB_piece = (uint32_t)((((wave * 64 + lane) % C::PPRB) ^ swizzle<C::PPRB>(ldB_row)) * 16);
    int ld_tile = vb / nqb, ld_qb = vb % nqb;
    int ld_c = 0, ld_stage = 0;
    typedef typename std::conditional<SAMPLE, uint64_t, uint32_t>::type OffA;   // a sampling pass addresses rows anywhere
    OffA offA[LA];
    uint32_t offB[LB];
    auto ld_setup = [&]() {
        const int64_t left = p.n_keys - ld_tile * tstride * TK;      // >= 1 rows in this tile
        const int last = left < TK ? (int)left - 1 : TK - 1;
        const int64_t tile_run = SAMPLE ? sample_tile_run(p, ld_tile, TK) : 0;
#pragma unroll
        for (int j = 0; j < LA; ++j) {
            int r = ldA_row + j * RSTEP_A;
            // (opaque in a sampling pass: the tile-independent part of the scattered-row arithmetic would otherwise be kept
            // per lane and load across the items, in registers that end up spilled)
            if constexpr (SAMPLE) asm volatile("" : "+v"(r));
            if constexpr (SAMPLE) offA[j] = (uint64_t)sample_row(p, tile_run, ld_tile, TK, r) * key_row_bytes + ldA_piece;
            else offA[j] = (uint32_t)(r < last ? r : last) * key_row_bytes + ldA_piece;
        }
        const int qlast = p.Q - 1 - ld_qb * TQ;
#pragma unroll
        for (int j = 0; j < LB; ++j) {
            const int r = ldB_row + j * RSTEP_B;
            offB[j] = (uint32_t)(ld_qb * TQ + (r < qlast ? r : qlast)) * qry_row_bytes + ldB_piece;
        }
    };
    auto issue_next = [&]() {
        unsigned char *sA = smem + ld_stage * C::STAGE_BYTES + wave * 1024;
        unsigned char *sB = sA + C::A_BYTES;
        const unsigned char *gA = static_cast<const unsigned char *>(p.keys) + (SAMPLE ? 0 : (size_t)(ld_tile * tstride) * TK * key_row_bytes) + (size_t)ld_c * RBA;
        const unsigned char *gB = static_cast<const unsigned char *>(p.queries) + (size_t)ld_c * RBB;
#pragma unroll
        for (int j = 0; j < LA; ++j)
            __builtin_amdgcn_global_load_lds((const void *)(gA + offA[j]), (lds_ptr)(sA + j * NW * 1024), 16, 0, 0);
#pragma unroll
        for (int j = 0; j < LB; ++j)
            __builtin_amdgcn_global_load_lds((const void *)(gB + offB[j]), (lds_ptr)(sB + j * NW * 1024), 16, 0, 0);
        if (++ld_c == NC) {
            ld_c = 0;
            ld_tile += step_tile;
            ld_qb += step_qb;
            if (ld_qb >= nqb) {
                ld_qb -= nqb;
                ++ld_tile;
            }
            if (ld_tile < p.n_tiles) ld_setup();
        }
        ld_stage = ld_stage + 1 == C::NSTAGE ? 0 : ld_stage + 1;
    };

    // ---- fragment addresses (bytes inside a stage) ----------------------------------------------
    const int rowA = wm * (TK / C::WM) + lrow;
    const int rowB = wn * (TQ / C::WN) + lrow;
    const int baseA = C::Q8 ? (rowA * RBA | (((2 * half) ^ swizzle<C::PPRA>(rowA)) << 4)) : (rowA * RBA | ((half ^ swizzle<C::PPRA>(rowA)) << 4));
    const int baseB = C::BMUL == 1 && !C::Q8 ? (rowB * RBB | ((half ^ swizzle<C::PPRB>(rowB)) << 4))
                                   : (rowB * RBB | (((2 * half) ^ swizzle<C::PPRB>(rowB)) << 4));

    f32x16 acc[IB][JB];
#pragma unroll
    for (int ib = 0; ib < IB; ++ib)
#pragma unroll
        for (int jb = 0; jb < JB; ++jb)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[ib][jb][i] = 0.f;

    if (total > 0) ld_setup();
#pragma unroll
    for (int s = 0; s < C::NSTAGE - 1; ++s)
        if (s < total) issue_next();

    int tile = vb / nqb, qb = vb % nqb;
    int c = 0, stage = 0;
    // per-item side data, fetched into registers while the item's last chunks are computed
    float my_invk = 0.f, my_invq = 0.f, my_lgain = 0.f;
    uint64_t my_tag = 0, my_thr64 = 0, my_qmask = 0;
    float my_thrp = __builtin_inff();
    const int aux_chunk = NC >= 2 ? NC - 2 : 0;

    for (int g = 0; g < total; ++g) {
        // chunk g has landed once at most the loads of the NSTAGE-2 younger chunks are outstanding
        if (g + (C::NSTAGE - 2) < total)
            __builtin_amdgcn_s_waitcnt(waitcnt_vm(C::VM_PER_CHUNK * (C::NSTAGE - 2)));
        else
            __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));
        bare_barrier();     // everyone's part of chunk g is in LDS; everyone is done reading chunk g-1
        if (g + (C::NSTAGE - 1) < total) issue_next();      // refills the buffer chunk g-1 was read from

        if (c == aux_chunk) {
            // unconditional loads from clamped / padded indices: nothing here is consumed before the epilogue,
            // so no wait on these loads lands inside the chunk loop
            if (tid < TK) {
                int64_t r = tile * tstride * TK + tid;
                r = r < p.n_keys ? r : p.n_keys - 1;
                if constexpr (SAMPLE) {
                    int rl = tid;
                    asm volatile("" : "+v"(rl));
                    r = sample_row(p, sample_tile_run(p, tile, TK), tile, TK, rl);
                }
                my_invk = p.inv_norm[r];
                if (filter) my_tag = p.tags[r];
                if constexpr (DRAW) my_lgain = p.draw.log_gain[r];
            }
            if (tid < TQ) {
                const int q = qb * TQ + tid;            // < qpad: invq, thr64 and thrp are padded arrays
                if (!SAMPLE || DRAW) my_invq = p.invq[q];      // (a sampling pass on scores runs before 1/|q| exists)
                if (!SAMPLE) {
                    my_thr64 = p.thr64[q];
                    my_thrp = p.thrp[q];
                }
                if (filter) my_qmask = p.qmask[q < p.Q ? q : p.Q - 1];
            }
        }

        // ---- contraction over this chunk --------------------------------------------------------
        {
            const unsigned char *sA = smem + stage * C::STAGE_BYTES;
            const unsigned char *sB = sA + C::A_BYTES;
#pragma unroll
            for (int kg = 0; kg < C::KG; ++kg) {
                typename Mma<C::KT>::PrepA a[IB];
                u32x4 b0[JB], b1[JB];
#pragma unroll
                for (int ib = 0; ib < IB; ++ib) {
                    if constexpr (C::Q8) {
                        a[ib].lo = *reinterpret_cast<const u32x4 *>(sA + ((baseA ^ (kg << 6)) + ib * 32 * RBA));
                        a[ib].hi = *reinterpret_cast<const u32x4 *>(sA + ((baseA ^ (kg << 6) ^ 16) + ib * 32 * RBA));
                    } else {
                        a[ib] = Mma<C::KT>::prepare(
                            *reinterpret_cast<const u32x4 *>(sA + ((baseA ^ (kg << 5)) + ib * 32 * RBA)));
                    }
                }
#pragma unroll
                for (int jb = 0; jb < JB; ++jb) {
                    if (C::BMUL == 1 && !C::Q8) {
                        b0[jb] = *reinterpret_cast<const u32x4 *>(sB + ((baseB ^ (kg << 5)) + jb * 32 * RBB));
                        b1[jb] = b0[jb];
                    } else {
                        b0[jb] = *reinterpret_cast<const u32x4 *>(sB + ((baseB ^ (kg << 6)) + jb * 32 * RBB));
                        b1[jb] = *reinterpret_cast<const u32x4 *>(sB + ((baseB ^ (kg << 6) ^ 16) + jb * 32 * RBB));
                    }
                }
#pragma unroll
                for (int ib = 0; ib < IB; ++ib)
#pragma unroll
                    for (int jb = 0; jb < JB; ++jb) Mma<C::KT>::run(acc[ib][jb], a[ib], b0[jb], b1[jb]);
            }
        }
        stage = stage + 1 == C::NSTAGE ? 0 : stage + 1;

        if (++c == NC) {
            // ---- epilogue of the item -----------------------------------------------------------
            // (the side-data buffers were last read in the previous epilogue, at least one barrier ago)
            if (tid < TK) {
                aux_invk[tid] = my_invk;
                aux_tag[tid] = my_tag;
                if constexpr (DRAW) aux_lgain[tid] = my_lgain;
            }
            if (tid < TQ) {
                aux_invq[tid] = my_invq;
                aux_qmask[tid] = my_qmask;
                aux_thr64[tid] = my_thr64;
                reinterpret_cast<float *>(smem + C::OFF_THRP)[tid] = my_thrp;
            }
            __builtin_amdgcn_s_waitcnt(waitcnt_lgkm0());
            bare_barrier();
            const int64_t row0 = SAMPLE ? sample_row0(p, tile, TK) : tile * tstride * TK;
            const EpiSide sd{aux_invk, aux_tag, reinterpret_cast<const float *>(smem + C::OFF_THRP), aux_invq, aux_thr64, aux_qmask, aux_lgain};
            if (SAMPLE && DRAW)
                sample_epilogue_draw<IB, JB>(acc, sd, filter, rowA - lrow, rowB, half, row0, qb * TQ, p,
                                             (int64_t)tile * C::GROUPS_PER_TILE + wm * 2 + half, sample_tile_run(p, tile, TK), TK);
            else if (SAMPLE)
                sample_epilogue<IB, JB, (IB * JB >= 8)>(acc, sd, filter, rowA - lrow, rowB, half, row0, qb * TQ, p,      // (128 accumulators: the search that needs few registers)
                                        (int64_t)tile * C::GROUPS_PER_TILE + wm * 2 + half, sample_tile_run(p, tile, TK), TK);
            else if (DRAW)
                main_epilogue_draw<IB, JB>(acc, sd, filter, rowA - lrow, rowB, half, row0, qb * TQ, p, my_region, wave_cnt, blockIdx.x * NW + wave);
            else
                main_epilogue<IB, JB, C::KEY_BYTES == 1>(acc, sd, filter, rowA - lrow, rowB, half, row0, qb * TQ, p, my_region, wave_cnt, blockIdx.x * NW + wave);
#pragma unroll
            for (int ib = 0; ib < IB; ++ib)
#pragma unroll
                for (int jb = 0; jb < JB; ++jb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) acc[ib][jb][i] = 0.f;
            c = 0;
            tile += step_tile;
            qb += step_qb;
            if (qb >= nqb) {
                qb -= nqb;
                ++tile;
            }
        }
    }

    if (!SAMPLE) flush_records(p, my_region, wave_cnt, blockIdx.x * NW + wave);      // what is left in the region
}

template <class C> hipError_t launch_scan_cfg(bool sample, int grid, const ScanArgs &a, hipStream_t s)
{
    // more than 64 KiB of dynamic LDS has to be requested explicitly, once per kernel
    static LdsAllowed allowed[4];
    const bool draw = a.draw.enabled != 0;
    auto *fn = draw ? (sample ? &kb_scan_kernel<C, true, true> : &kb_scan_kernel<C, false, true>)
                    : (sample ? &kb_scan_kernel<C, true, false> : &kb_scan_kernel<C, false, false>);
    const int which = (draw ? 2 : 0) + (sample ? 1 : 0);
    if (hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(fn), allowed[which], C::SMEM_BYTES); e != hipSuccess) return e;
    hipExtLaunchKernelGGL(fn, dim3(grid), dim3(C::THREADS), C::SMEM_BYTES, s, scan_timing.start, scan_timing.stop, 0, a);
    return hipGetLastError();
}

}  // namespace kbi
