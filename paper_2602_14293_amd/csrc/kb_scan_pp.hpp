// The large-batch scan kernel: 8 wavefronts per workgroup in two groups that alternate between
// "fetch fragments from LDS" and "issue MFMAs", so that each SIMD always has one wavefront feeding its
// matrix core while the other refills its operand registers (gfx950 only).
//
// Tile: 256 key rows x TQ queries x all of d per work item, one workgroup (512 threads) per compute unit.
// Wave w: SIMD w % 4, group w / 4.  Rows [64 * (w % 4), +64) of the tile, query columns
// [(TQ/2) * (w / 4), +TQ/2): every SIMD hosts one wave of each group.  Work decomposition, operand
// layout (S^T = K * Q^T, a lane owns one query column), swizzled direct-to-LDS staging, candidate words,
// sampling and threshold filter are those of kb_scan.hpp; what differs is the schedule:
//
//   barrier index      0     1      2      3      4
//   group 0            | L0  |  C0  |  L1  |  C1  | ...          L = 12 x ds_read_b128 (one d-chunk of
//   group 1            |  -  |  L0  |  C0  |  L1  | ...              fragments) + the wave's share of the
//                                                                    direct-to-LDS loads of chunk c+D
//                                                                C = 16 MFMAs from registers
// Both groups run the same instruction stream, shifted by one barrier.  The epilogue of a tile runs at
// the start of the next L phase, i.e. while the other group's MFMAs keep the matrix cores busy.
// Per-tile side data (1/|k|, tags) and per-query data (thresholds, 1/|q|, mask words) arrive by
// direct-to-LDS loads as well, double-buffered by item parity.
#pragma once
#include "kb_scan.hpp"

namespace kbi {

template <int KT_, int TQ_, int NSA_, int NSB_> struct PPCfg {
    static constexpr int KT = KT_, TQ = TQ_, NSA = NSA_, NSB = NSB_;     // ring depths: key chunks, query chunks
    static constexpr int TK = 256, THREADS = 512, NW = 8, RBA = 64;
    static constexpr int KEY_BYTES = KeyTraits<KT>::KEY_BYTES, QRY_BYTES = KeyTraits<KT>::QRY_BYTES;
    static constexpr int BMUL = QRY_BYTES / KEY_BYTES;
    static constexpr int RBB = RBA * BMUL;
    static constexpr int PPRA = RBA / 16, PPRB = RBB / 16;
    static constexpr int KG = RBA / 32;
    static constexpr int IB = 2, JB = TQ / 2 / 32;
    static constexpr int A_BYTES = TK * RBA, B_BYTES = TQ * RBB;
    // Even waves load key chunks, odd waves load query chunks.  vmcnt counts per wave and completes in order, so
    // separate issuers let the key stream (HBM latency) run deeper than the query stream (L2 hits).
    static constexpr int LA = A_BYTES / 1024 / 4, LB = B_BYTES / 1024 / 4;      // load instructions per loading wave per chunk
    static constexpr int DA = NSA - 1, DB = NSB - 1;                             // prefetch distances in chunks
    static constexpr int OFF_B = NSA * A_BYTES;
    // side data, two copies (item parity)
    static constexpr int AUX_INVK = 0;                       // float  [TK]
    static constexpr int AUX_TAG = AUX_INVK + TK * 4;        // uint64 [TK]
    static constexpr int AUX_THRP = AUX_TAG + TK * 8;        // float  [TQ]
    static constexpr int AUX_INVQ = AUX_THRP + TQ * 4;       // float  [TQ]
    static constexpr int AUX_THR64 = AUX_INVQ + TQ * 4;      // uint64 [TQ]
    static constexpr int AUX_QMASK = AUX_THR64 + TQ * 8;     // uint64 [TQ]
    static constexpr int AUX_BYTES = AUX_QMASK + TQ * 8;
    static constexpr int OFF_AUX = NSA * A_BYTES + NSB * B_BYTES;
    static constexpr int OFF_CNT = OFF_AUX + 2 * AUX_BYTES;
    static constexpr int SMEM_BYTES = OFF_CNT + 16;
    static constexpr int GROUPS_PER_TILE = 8;                // sampling groups: 4 row blocks x 2 lane halves
    static_assert(TQ == 256, "query block of 256");
    static_assert(A_BYTES % 4096 == 0 && B_BYTES % 4096 == 0, "four waves share each chunk evenly");
    static_assert(NSA >= 3 && NSB >= 3, "a chunk is awaited up to one iteration before it is fetched");
    static_assert(SMEM_BYTES <= 160 * 1024, "LDS budget");
    static_assert(LA * (DA - 1) < 64 && LB * (DB - 1) < 64, "vmcnt is a 6-bit counter");
    static_assert((TQ * 4) % 1024 == 0, "per-query side data is loaded 1 KiB per wave instruction");
};

template <class C, bool SAMPLE>
__global__ __launch_bounds__(512, 1) void kb_scan_pp_kernel(ScanArgs p)
{
    constexpr int TK = C::TK, TQ = C::TQ, RBA = C::RBA, RBB = C::RBB, IB = C::IB, JB = C::JB, NW = C::NW;
    constexpr int LA = C::LA, LB = C::LB, DA = C::DA, DB = C::DB;
    constexpr int RSTEP_A = 256 / C::PPRA, RSTEP_B = 256 / C::PPRB;      // rows between a loading wave's instructions
    static_assert(RSTEP_A % 32 == 0 && RSTEP_B % 32 == 0, "the swizzle must not change between instructions");
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    typedef __attribute__((address_space(3))) void *lds_ptr;

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

    // ---- the load stream of this wave: key chunks (role 0) or query chunks (role 1) ---------------
    const int role = wave & 1, ridx = wave >> 1;
    const int ld_row = (ridx * 64 + lane) / (role ? C::PPRB : C::PPRA);
    const uint32_t ld_piece = role ? (uint32_t)((((ridx * 64 + lane) % C::PPRB) ^ swizzle<C::PPRB>(ld_row)) * 16)
                                   : (uint32_t)((((ridx * 64 + lane) % C::PPRA) ^ swizzle<C::PPRA>(ld_row)) * 16);
    int ld_tile = vb / nqb, ld_qb = vb % nqb;
    int ld_c = 0, ld_stage = 0, ld_par = 0;
    constexpr int LMAX = LA > LB ? LA : LB;
    uint32_t off[LMAX];
    auto ld_setup = [&]() {
        if (role == 0) {
            const int64_t left = p.n_keys - ld_tile * tstride * TK;
            const int last = left < TK ? (int)left - 1 : TK - 1;
#pragma unroll
            for (int j = 0; j < LA; ++j) {
                const int r = ld_row + j * RSTEP_A;
                off[j] = (uint32_t)(r < last ? r : last) * key_row_bytes + ld_piece;
            }
        } else {
            const int qlast = p.Q - 1 - ld_qb * TQ;
#pragma unroll
            for (int j = 0; j < LB; ++j) {
                const int r = ld_row + j * RSTEP_B;
                off[j] = (uint32_t)(ld_qb * TQ + (r < qlast ? r : qlast)) * qry_row_bytes + ld_piece;
            }
        }
    };
    // side data of the item the load stream is at: 4-byte loads with clamped rows for the caller's arrays
    // (inv_norm, tags), 16-byte loads for the library's padded per-query arrays
    auto issue_aux = [&]() {
        unsigned char *aux = smem + C::OFF_AUX + ld_par * C::AUX_BYTES;
        const int64_t row0 = ld_tile * tstride * TK;
        if (wave < 4) {
            int64_t r = row0 + wave * 64 + lane;
            r = r < p.n_keys ? r : p.n_keys - 1;
            __builtin_amdgcn_global_load_lds((const void *)(p.inv_norm + r), (lds_ptr)(aux + C::AUX_INVK + wave * 256), 4, 0, 0);
        }
        if (filter) {
            // tags as dwords: wave w covers dwords [64w, 64w+64) = rows [32w, 32w+32)
            int64_t r = row0 + wave * 32 + (lane >> 1);
            r = r < p.n_keys ? r : p.n_keys - 1;
            __builtin_amdgcn_global_load_lds((const void *)(reinterpret_cast<const uint32_t *>(p.tags + r) + (lane & 1)),
                                             (lds_ptr)(aux + C::AUX_TAG + wave * 256), 4, 0, 0);
        }
        const int q0 = ld_qb * TQ;
        constexpr int NI4 = TQ * 4 / 1024, NI8 = TQ * 8 / 1024;     // wave instructions per array
        // wave-uniform dispatch of the per-query arrays over the eight waves
        int slot = wave;
        if (slot < NI4) {
            __builtin_amdgcn_global_load_lds((const void *)(p.invq + q0 + slot * 256 + lane * 4),
                                             (lds_ptr)(aux + C::AUX_INVQ + slot * 1024), 16, 0, 0);
            if (!SAMPLE)
                __builtin_amdgcn_global_load_lds((const void *)(p.thrp + q0 + slot * 256 + lane * 4),
                                                 (lds_ptr)(aux + C::AUX_THRP + slot * 1024), 16, 0, 0);
        }
        slot = wave - 2;
        if (slot >= 0 && slot < NI8) {
            if (!SAMPLE)
                __builtin_amdgcn_global_load_lds((const void *)(p.thr64 + q0 + slot * 128 + lane * 2),
                                                 (lds_ptr)(aux + C::AUX_THR64 + slot * 1024), 16, 0, 0);
        }
        slot = wave - 4;
        if (slot >= 0 && slot < NI8 && filter)
            __builtin_amdgcn_global_load_lds((const void *)(p.qmask_pad + q0 + slot * 128 + lane * 2),
                                             (lds_ptr)(aux + C::AUX_QMASK + slot * 1024), 16, 0, 0);
    };
    // One chunk of this wave's stream = LD loads; issue_one(j) is called LD times (interleaved with the MFMAs of
    // the compute phase), then issue_end() advances the stream.
    auto issue_one = [&](int j) {
        if (j == 0 && ld_c == 0) issue_aux();
        if (role == 0) {
            if (j < LA) {
                unsigned char *dst = smem + ld_stage * C::A_BYTES + ridx * 1024;
                const unsigned char *g = static_cast<const unsigned char *>(p.keys) + (size_t)(ld_tile * tstride) * TK * key_row_bytes + (size_t)ld_c * RBA;
                __builtin_amdgcn_global_load_lds((const void *)(g + off[j]), (lds_ptr)(dst + j * 4096), 16, 0, 0);
            }
        } else {
            if (j < LB) {
                unsigned char *dst = smem + C::OFF_B + ld_stage * C::B_BYTES + ridx * 1024;
                const unsigned char *g = static_cast<const unsigned char *>(p.queries) + (size_t)ld_c * RBB;
                __builtin_amdgcn_global_load_lds((const void *)(g + off[j]), (lds_ptr)(dst + j * 4096), 16, 0, 0);
            }
        }
    };
    auto issue_end = [&]() {
        ld_stage = ld_stage + 1 == (role ? C::NSB : C::NSA) ? 0 : ld_stage + 1;
        if (++ld_c == NC) {
            ld_c = 0;
            ld_par ^= 1;
            ld_tile += step_tile;
            ld_qb += step_qb;
            if (ld_qb >= nqb) {
                ld_qb -= nqb;
                ++ld_tile;
            }
            if (ld_tile < p.n_tiles) ld_setup();
        }
    };
    auto issue_next = [&]() {
#pragma unroll
        for (int j = 0; j < LMAX; ++j) issue_one(j);
        issue_end();
    };
    // my share of a chunk has landed once at most the loads of `younger` younger chunks of my stream are outstanding
    // (younger = 0: everything has landed); compile-time immediates, so the cases are spelled out
    auto wait_landed = [&](int younger) {
        const int n = younger * (role ? LB : LA);
        if (n <= 0) __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));
        else if (n == LA * (DA - 1) && role == 0) __builtin_amdgcn_s_waitcnt(waitcnt_vm(LA * (DA - 1)));
        else if (n == LA * (DA - 2) && role == 0) __builtin_amdgcn_s_waitcnt(waitcnt_vm(LA * (DA - 2) > 0 ? LA * (DA - 2) : 0));
        else if (n == LB * (DB - 1) && role == 1) __builtin_amdgcn_s_waitcnt(waitcnt_vm(LB * (DB - 1)));
        else if (n == LB * (DB - 2) && role == 1) __builtin_amdgcn_s_waitcnt(waitcnt_vm(LB * (DB - 2) > 0 ? LB * (DB - 2) : 0));
        else __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));
    };
    const int D = role ? DB : DA;

    // ---- fragment addresses ----------------------------------------------------------------------
    const int rowA = wm * 64 + lrow;
    const int rowB = group * (TQ / 2) + lrow;
    const int baseA = rowA * RBA | ((half ^ swizzle<C::PPRA>(rowA)) << 4);
    const int baseB = C::BMUL == 1 ? (rowB * RBB | ((half ^ swizzle<C::PPRB>(rowB)) << 4))
                                   : (rowB * RBB | (((2 * half) ^ swizzle<C::PPRB>(rowB)) << 4));

    f32x16 acc[IB][JB];
#pragma unroll
    for (int ib = 0; ib < IB; ++ib)
#pragma unroll
        for (int jb = 0; jb < JB; ++jb)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[ib][jb][i] = 0.f;

    // ---- the epilogue of one item (runs at the start of the following fetch phase) ----------------
    auto epilogue = [&](int tile, int qb, int par) {
        const unsigned char *aux = smem + C::OFF_AUX + par * C::AUX_BYTES;
        const float *aux_invk = reinterpret_cast<const float *>(aux + C::AUX_INVK);
        const uint64_t *aux_tag = reinterpret_cast<const uint64_t *>(aux + C::AUX_TAG);
        const float *aux_thrp = reinterpret_cast<const float *>(aux + C::AUX_THRP);
        const float *aux_invq = reinterpret_cast<const float *>(aux + C::AUX_INVQ);
        const uint64_t *aux_thr64 = reinterpret_cast<const uint64_t *>(aux + C::AUX_THR64);
        const uint64_t *aux_qmask = reinterpret_cast<const uint64_t *>(aux + C::AUX_QMASK);
        const int64_t row0 = tile * tstride * TK;
        const EpiSide sd{aux_invk, aux_tag, aux_thrp, aux_invq, aux_thr64, aux_qmask};
        if (SAMPLE)
            sample_epilogue<IB, JB>(acc, sd, filter, wm * 64, rowB, half, row0, qb * TQ, p,
                                    (int64_t)tile * C::GROUPS_PER_TILE + wm * 2 + half);
        else
            main_epilogue<IB, JB>(acc, sd, filter, wm * 64, rowB, half, row0, qb * TQ, p, my_region, wave_cnt);
#pragma unroll
        for (int ib = 0; ib < IB; ++ib)
#pragma unroll
            for (int jb = 0; jb < JB; ++jb)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[ib][jb][i] = 0.f;
    };

    // ---- prologue: D chunks in flight per stream, chunk 0 landed -----------------------------------
    if (total > 0) ld_setup();
    for (int s = 0; s < D; ++s)
        if (s < total) issue_next();
    wait_landed(total >= D ? D - 1 : 0);
    __builtin_amdgcn_s_waitcnt(waitcnt_lgkm0());
    bare_barrier();                         // barrier 0
    if (group == 1) bare_barrier();         // group 1 runs one barrier behind

    int tile = vb / nqb, qb = vb % nqb, par = 0;
    int c = 0, stageA = 0, stageB = 0;
    bool pending = false;                   // an item is complete and waits for its epilogue
    int e_tile = 0, e_qb = 0, e_par = 0;

    for (int g = 0; g < total; ++g) {
        // ================= fetch phase =================
        if (pending) {
            epilogue(e_tile, e_qb, e_par);
            pending = false;
        }
        // 12 fragment reads (LDS-bandwidth bound: four waves x 12 KiB per phase) with this wave's loads of chunk
        // g+D in between: a direct-to-LDS load holds the issuing wave for 50-90 cycles while the texture-address
        // unit takes its 64 addresses, and the LDS keeps serving the reads already issued meanwhile.  The loads
        // refill the ring slot of chunk g-1, which both groups have fetched.
        typename Mma<C::KT>::PrepA fa[C::KG][IB];
        u32x4 fb0[C::KG][JB], fb1[C::KG][JB];
        {
            const unsigned char *sA = smem + stageA * C::A_BYTES;
            const unsigned char *sB = smem + C::OFF_B + stageB * C::B_BYTES;
            constexpr int PER_KG = IB + JB, NR = C::KG * PER_KG, EVERY = NR / LMAX;
            static_assert(NR % LMAX == 0, "loads spread evenly over the fragment reads");
            const bool more = g + D < total;
#pragma unroll
            for (int r = 0; r < NR; ++r) {
                const int kg = r / PER_KG, x = r % PER_KG;
                if (x < IB) {
                    fa[kg][x] = Mma<C::KT>::prepare(*reinterpret_cast<const u32x4 *>(sA + ((baseA ^ (kg << 5)) + x * 32 * RBA)));
                } else {
                    const int jb = x - IB;
                    if (C::BMUL == 1) {
                        fb0[kg][jb] = *reinterpret_cast<const u32x4 *>(sB + ((baseB ^ (kg << 5)) + jb * 32 * RBB));
                        fb1[kg][jb] = fb0[kg][jb];
                    } else {
                        fb0[kg][jb] = *reinterpret_cast<const u32x4 *>(sB + ((baseB ^ (kg << 6)) + jb * 32 * RBB));
                        fb1[kg][jb] = *reinterpret_cast<const u32x4 *>(sB + ((baseB ^ (kg << 6) ^ 16) + jb * 32 * RBB));
                    }
                }
                if ((r + 1) % EVERY == 0) {
                    __builtin_amdgcn_sched_barrier(0);
                    if (more) issue_one((r + 1) / EVERY - 1);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            if (more) issue_end();
        }
        // My share of chunk g+1 must have landed before the next barrier (the other group fetches it first); I have
        // issued chunks up to g+D.  The side data of the item being computed is older than every chunk load in flight.
        wait_landed(g + D < total ? D - 1 : 0);
        __builtin_amdgcn_s_waitcnt(waitcnt_lgkm0());
        __builtin_amdgcn_sched_barrier(0);
        bare_barrier();
        __builtin_amdgcn_sched_barrier(0);

        // ================= MFMA phase: 16 MFMAs from registers =================
        __builtin_amdgcn_s_setprio(1);
#pragma unroll
        for (int kg = 0; kg < C::KG; ++kg)
#pragma unroll
            for (int ib = 0; ib < IB; ++ib)
#pragma unroll
                for (int jb = 0; jb < JB; ++jb) Mma<C::KT>::run(acc[ib][jb], fa[kg][ib], fb0[kg][jb], fb1[kg][jb]);
        __builtin_amdgcn_s_setprio(0);
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
        __builtin_amdgcn_sched_barrier(0);
        bare_barrier();
        __builtin_amdgcn_sched_barrier(0);
    }
    if (pending) epilogue(e_tile, e_qb, e_par);
    if (group == 0) bare_barrier();         // matches the extra barrier group 1 took at the start

    if (!SAMPLE && lane == 0) {
        const uint32_t cap = (uint32_t)p.region_cap;
        p.region_cnt[blockIdx.x * NW + wave] = wave_cnt < cap ? wave_cnt : cap;
    }
}

template <class C> hipError_t launch_scan_pp_cfg(bool sample, int grid, const ScanArgs &a, hipStream_t s)
{
    static bool attr_done[2] = {false, false};
    auto *fn = sample ? &kb_scan_pp_kernel<C, true> : &kb_scan_pp_kernel<C, false>;
    if (!attr_done[sample]) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(fn), hipFuncAttributeMaxDynamicSharedMemorySize, C::SMEM_BYTES);
        if (e != hipSuccess) return e;
        attr_done[sample] = true;
    }
    hipLaunchKernelGGL(fn, dim3(grid), dim3(C::THREADS), C::SMEM_BYTES, s, a);
    return hipGetLastError();
}

}  // namespace kbi
