// The large-batch scan kernel, register-tile version: four wavefronts per workgroup, one per SIMD, each
// owning a 128-key x 128-query accumulator tile (256 accumulator registers per lane) and software-pipelining
// its own LDS fragment reads and direct-to-LDS loads under its MFMAs (gfx950 only).
//
// Why this shape.  Per compute unit the LDS serves about 128 bytes per clock and the texture-address path
// about 64; a 256 x 256 x 32 contraction step takes 1024 matrix-core clocks.  With 64 x 128 wave tiles the
// eight waves read 96 KiB of fragments per step (LDS about 100 % busy once the 32 KiB of incoming chunk data
// are added); with 128 x 128 wave tiles four waves read 64 KiB (about 75 %).  The price is that nothing
// overlaps for free any more: a wave has no partner on its SIMD, so the instruction order below is the
// pipeline.
//
// Per d-chunk of 64 bytes per row (two k-groups): step (c,0) issues the 16 MFMAs of k-group 0 from fragment
// buffer 0 while reading k-group 1 of the same chunk into buffer 1; the mid-chunk barrier publishes chunk
// c+1 (every wave has waited for its own loads) and retires chunk c; step (c,1) issues the MFMAs of k-group 1
// while reading k-group 0 of chunk c+1 into buffer 0.  The wave's eight direct-to-LDS loads of chunk
// c + NS - 1 (waves 0,1: key rows; waves 2,3: query rows) are spread over the two steps and refill the ring
// slot of chunk c-1.  Work decomposition, swizzle, candidate words, sampling and threshold filter are those
// of kb_scan.hpp.
#pragma once
#include "kb_scan.hpp"

namespace kbi {

// MFMA with the accumulator pinned to the accumulation register file.  With 256 accumulator registers per
// lane the register allocator otherwise shuffles tiles between the two files inside the loop.  The asm hides
// the instruction from the hazard recognizer: callers keep dependent uses of an accumulator at least 16
// MFMAs apart and put explicit no-ops before reading accumulators with vector instructions.
__device__ inline void mfma_acc(f32x16 &c, const u32x4 &a, const u32x4 &b)
{
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(c) : "v"(a), "v"(b));
}

// First MFMA of an item: C = 0 as an inline constant, so accumulators are never written by vector moves.
__device__ inline void mfma_first(f32x16 &c, const u32x4 &a, const u32x4 &b)
{
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=a"(c) : "v"(a), "v"(b));
}

template <int KT_, int NSA_, int NSB_> struct BigCfg {
    static constexpr int KT = KT_, NSA = NSA_, NSB = NSB_;
    static constexpr int TK = 256, TQ = 256, THREADS = 256, NW = 4, RBA = 64;
    static constexpr int KEY_BYTES = KeyTraits<KT>::KEY_BYTES, QRY_BYTES = KeyTraits<KT>::QRY_BYTES;
    static constexpr int BMUL = QRY_BYTES / KEY_BYTES;
    static constexpr int RBB = RBA * BMUL;
    static constexpr int PPRA = RBA / 16, PPRB = RBB / 16;
    static constexpr int IB = 4, JB = 4;
    static constexpr int A_BYTES = TK * RBA, B_BYTES = TQ * RBB;
    static constexpr int LA = A_BYTES / 1024 / 2, LB = B_BYTES / 1024 / 2;      // loads per loading wave per chunk
    static constexpr int OFF_B = NSA * A_BYTES;
    static constexpr int AUX_INVK = 0;
    static constexpr int AUX_TAG = AUX_INVK + TK * 4;
    static constexpr int AUX_THRP = AUX_TAG + TK * 8;
    static constexpr int AUX_INVQ = AUX_THRP + TQ * 4;
    static constexpr int AUX_THR64 = AUX_INVQ + TQ * 4;
    static constexpr int AUX_QMASK = AUX_THR64 + TQ * 8;
    static constexpr int AUX_BYTES = AUX_QMASK + TQ * 8;
    static constexpr int OFF_AUX = NSA * A_BYTES + NSB * B_BYTES;
    static constexpr int SMEM_BYTES = OFF_AUX + 2 * AUX_BYTES;
    static constexpr int GROUPS_PER_TILE = 4;                // sampling groups: 2 row blocks x 2 lane halves
    static_assert(BMUL == 1, "same element width for keys and queries");
    static_assert(NSA >= 3 && NSB >= 3, "ring depth");
    static_assert(LA == 8 && LB == 8, "eight loads per wave per chunk, four per k-group step");
    static_assert(SMEM_BYTES <= 160 * 1024, "LDS budget");
    static_assert(8 * (NSA - 3) + 4 < 64 && 8 * (NSB - 3) + 4 < 64, "vmcnt is a 6-bit counter");
};

template <class C, bool SAMPLE>
__global__ __launch_bounds__(256, 1) void kb_scan_big_kernel(ScanArgs p)
{
    constexpr int TK = C::TK, TQ = C::TQ, RBA = C::RBA, RBB = C::RBB, IB = C::IB, JB = C::JB, NW = C::NW;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    typedef __attribute__((address_space(3))) void *lds_ptr;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;
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
    uint32_t wave_cnt = 0;

    // ---- the load stream of this wave: key chunks (waves 0,1) or query chunks (waves 2,3) -------------
    const int role = wave >> 1, ridx = wave & 1;
    const int NS = role ? C::NSB : C::NSA;
    const int ld_row = (ridx * 64 + lane) / (role ? C::PPRB : C::PPRA);
    const uint32_t ld_piece = role ? (uint32_t)((((ridx * 64 + lane) % C::PPRB) ^ swizzle<C::PPRB>(ld_row)) * 16)
                                   : (uint32_t)((((ridx * 64 + lane) % C::PPRA) ^ swizzle<C::PPRA>(ld_row)) * 16);
    constexpr int RSTEP = 2 * 64 / C::PPRA;          // rows between a loading wave's instructions (PPRA == PPRB)
    static_assert(C::PPRA == C::PPRB && RSTEP % 32 == 0, "the swizzle must not change between instructions");
    int ld_tile = vb / nqb, ld_qb = vb % nqb;
    int ld_c = 0, ld_stage = 0, ld_par = 0, ld_chunk = 0;        // ld_chunk: index of the chunk the stream is at
    uint32_t off[8];
    auto ld_setup = [&]() {
        if (role == 0) {
            const int64_t left = p.n_keys - ld_tile * tstride * TK;
            const int last = left < TK ? (int)left - 1 : TK - 1;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int r = ld_row + j * RSTEP;
                off[j] = (uint32_t)(r < last ? r : last) * key_row_bytes + ld_piece;
            }
        } else {
            const int qlast = p.Q - 1 - ld_qb * TQ;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int r = ld_row + j * RSTEP;
                off[j] = (uint32_t)(ld_qb * TQ + (r < qlast ? r : qlast)) * qry_row_bytes + ld_piece;
            }
        }
    };
    auto issue_aux = [&]() {
        unsigned char *aux = smem + C::OFF_AUX + ld_par * C::AUX_BYTES;
        const int64_t row0 = ld_tile * tstride * TK;
        {
            int64_t r = row0 + wave * 64 + lane;
            r = r < p.n_keys ? r : p.n_keys - 1;
            __builtin_amdgcn_global_load_lds((const void *)(p.inv_norm + r), (lds_ptr)(aux + C::AUX_INVK + wave * 256), 4, 0, 0);
        }
        if (filter) {
#pragma unroll
            for (int h2 = 0; h2 < 2; ++h2) {        // tags as dwords: instruction i covers rows [32 i, 32 i + 32)
                const int i = wave * 2 + h2;
                int64_t r = row0 + i * 32 + (lane >> 1);
                r = r < p.n_keys ? r : p.n_keys - 1;
                __builtin_amdgcn_global_load_lds((const void *)(reinterpret_cast<const uint32_t *>(p.tags + r) + (lane & 1)),
                                                 (lds_ptr)(aux + C::AUX_TAG + i * 256), 4, 0, 0);
            }
        }
        const int q0 = ld_qb * TQ;
        if (wave == 0) {
            __builtin_amdgcn_global_load_lds((const void *)(p.invq + q0 + lane * 4), (lds_ptr)(aux + C::AUX_INVQ), 16, 0, 0);
            if (!SAMPLE)
                __builtin_amdgcn_global_load_lds((const void *)(p.thrp + q0 + lane * 4), (lds_ptr)(aux + C::AUX_THRP), 16, 0, 0);
        } else if (wave == 1) {
            if (!SAMPLE) {
                __builtin_amdgcn_global_load_lds((const void *)(p.thr64 + q0 + lane * 2), (lds_ptr)(aux + C::AUX_THR64), 16, 0, 0);
                __builtin_amdgcn_global_load_lds((const void *)(p.thr64 + q0 + 128 + lane * 2), (lds_ptr)(aux + C::AUX_THR64 + 1024), 16, 0, 0);
            }
        } else if (wave == 2) {
            if (filter) {
                __builtin_amdgcn_global_load_lds((const void *)(p.qmask_pad + q0 + lane * 2), (lds_ptr)(aux + C::AUX_QMASK), 16, 0, 0);
                __builtin_amdgcn_global_load_lds((const void *)(p.qmask_pad + q0 + 128 + lane * 2), (lds_ptr)(aux + C::AUX_QMASK + 1024), 16, 0, 0);
            }
        }
    };
    auto issue_one = [&](int j) {
        if (j == 0 && ld_c == 0) issue_aux();
        if (role == 0) {
            unsigned char *dst = smem + ld_stage * C::A_BYTES + ridx * 1024;
            const unsigned char *g = static_cast<const unsigned char *>(p.keys) + (size_t)(ld_tile * tstride) * TK * key_row_bytes + (size_t)ld_c * RBA;
            __builtin_amdgcn_global_load_lds((const void *)(g + off[j]), (lds_ptr)(dst + j * 2048), 16, 0, 0);
        } else {
            unsigned char *dst = smem + C::OFF_B + ld_stage * C::B_BYTES + ridx * 1024;
            const unsigned char *g = static_cast<const unsigned char *>(p.queries) + (size_t)ld_c * RBB;
            __builtin_amdgcn_global_load_lds((const void *)(g + off[j]), (lds_ptr)(dst + j * 2048), 16, 0, 0);
        }
    };
    auto issue_end = [&]() {
        ld_stage = ld_stage + 1 == NS ? 0 : ld_stage + 1;
        ++ld_chunk;
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
    // at the mid-chunk barrier of chunk c: my share of chunk c+1 has landed once at most the loads of the younger
    // chunks (c+2 .. c+NS-2 in full, half of c+NS-1) are outstanding
    auto wait_mid = [&](bool full_depth) {
        if (!full_depth) __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));
        else if (role == 0) __builtin_amdgcn_s_waitcnt(waitcnt_vm(8 * (C::NSA - 3) + 4));
        else __builtin_amdgcn_s_waitcnt(waitcnt_vm(8 * (C::NSB - 3) + 4));
    };

    // ---- fragment addresses ----------------------------------------------------------------------
    const int rowA = wm * 128 + lrow, rowB = wn * 128 + lrow;
    const int baseA = rowA * RBA | ((half ^ swizzle<C::PPRA>(rowA)) << 4);
    const int baseB = rowB * RBB | ((half ^ swizzle<C::PPRB>(rowB)) << 4);

    // Accumulators are only ever written by the MFMA asm (accumulation registers); the first MFMA of an item has
    // C = 0.  The empty asm gives them a defined (arbitrary) value for the compiler without emitting anything.
    f32x16 acc[IB][JB];
#pragma unroll
    for (int ib = 0; ib < IB; ++ib)
#pragma unroll
        for (int jb = 0; jb < JB; ++jb) asm volatile("" : "=a"(acc[ib][jb]));

    auto epilogue = [&](int tile, int qb, int par) {
        const unsigned char *aux = smem + C::OFF_AUX + par * C::AUX_BYTES;
        const EpiSide sd{reinterpret_cast<const float *>(aux + C::AUX_INVK), reinterpret_cast<const uint64_t *>(aux + C::AUX_TAG),
                         reinterpret_cast<const float *>(aux + C::AUX_THRP), reinterpret_cast<const float *>(aux + C::AUX_INVQ),
                         reinterpret_cast<const uint64_t *>(aux + C::AUX_THR64), reinterpret_cast<const uint64_t *>(aux + C::AUX_QMASK)};
        const int64_t row0 = tile * tstride * TK;
        if (SAMPLE) {
#pragma unroll
            for (int jb = 0; jb < JB; ++jb) {
                float best = -__builtin_inff();
                int best_rl = -1;
                const uint64_t qm = filter ? sd.qmask[rowB + jb * 32] : 0ull;
#pragma unroll
                for (int ib = 0; ib < IB; ++ib) {
                    __builtin_amdgcn_sched_barrier(0);
                    f32x16 blk = acc[ib][jb];
                    asm volatile("" : "+v"(blk));
                    sample_block(blk, wm * 128 + ib * 32 + 4 * half, sd, filter, qm, row0, p.n_keys, best, best_rl);
                    __builtin_amdgcn_sched_barrier(0);
                }
                sample_store(best, best_rl, rowB + jb * 32, sd, row0, qb * TQ, p, (int64_t)tile * C::GROUPS_PER_TILE + wm * 2 + half);
            }
        } else {
            // one 32x32 block at a time: copy its 16 accumulators to vector registers, filter, next (the fences
            // keep the compiler from hoisting all 256 copies to the front)
            float thrp[JB];
#pragma unroll
            for (int jb = 0; jb < JB; ++jb) thrp[jb] = sd.thrp[rowB + jb * 32];
#pragma unroll
            for (int ib = 0; ib < IB; ++ib) {
                const EpiRows rw = load_rows(sd, wm * 128 + ib * 32 + 4 * half);
#pragma unroll
                for (int jb = 0; jb < JB; ++jb) {
                    __builtin_amdgcn_sched_barrier(0);
                    f32x16 blk = acc[ib][jb];
                    asm volatile("" : "+v"(blk));
                    main_block(blk, rw, thrp[jb], rowB + jb * 32, sd, filter, row0, qb * TQ, p, my_region, wave_cnt);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
    };

    // read the 8 fragments of k-group kg of the chunk in ring slots (sa, sb), one at a time (index r = 0..7)
    u32x4 fa[2][IB], fb[2][JB];
    auto read_frag = [&](int buf, int sa, int sb, int kg, int r) {
        if (r < IB)
            fa[buf][r] = *reinterpret_cast<const u32x4 *>(smem + sa * C::A_BYTES + ((baseA ^ (kg << 5)) + r * 32 * RBA));
        else
            fb[buf][r - IB] = *reinterpret_cast<const u32x4 *>(smem + C::OFF_B + sb * C::B_BYTES + ((baseB ^ (kg << 5)) + (r - IB) * 32 * RBB));
    };

    // ---- prologue: NS-1 chunks in flight per stream, chunk 0 landed, fragments of (0,0) in buffer 0 ----
    if (total > 0) ld_setup();
    for (int s = 0; s < NS - 1; ++s)
        if (s < total) {
#pragma unroll
            for (int j = 0; j < 8; ++j) issue_one(j);
            issue_end();
        }
    if (total >= NS - 1) {
        if (role == 0) __builtin_amdgcn_s_waitcnt(waitcnt_vm(8 * (C::NSA - 2)));
        else __builtin_amdgcn_s_waitcnt(waitcnt_vm(8 * (C::NSB - 2)));
    } else {
        __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));
    }
    __builtin_amdgcn_s_waitcnt(waitcnt_lgkm0());
    bare_barrier();
    if (total > 0) {
#pragma unroll
        for (int r = 0; r < 8; ++r) read_frag(0, 0, 0, 0, r);
    }

    int tile = vb / nqb, qb = vb % nqb, par = 0;
    int c = 0, sA = 0, sB = 0;

    for (int g = 0; g < total; ++g) {
        const bool more = ld_chunk < total;              // this iteration issues the loads of chunk ld_chunk = g + NS - 1
        const int sA1 = sA + 1 == C::NSA ? 0 : sA + 1, sB1 = sB + 1 == C::NSB ? 0 : sB + 1;
        // ---------------- step (g, 0): MFMAs from buffer 0, fragments (g, 1) into buffer 1 ----------------
        if (c == 0) {
#pragma unroll
            for (int m = 0; m < 16; ++m) {
                const int ib = m / JB, jb = m % JB;
                mfma_first(acc[ib][jb], fa[0][ib], fb[0][jb]);
                if (m % 2 == 1) read_frag(1, sA, sB, 1, m / 2);
                if (m % 4 == 3 && more) issue_one(m / 4);
                __builtin_amdgcn_sched_barrier(0);
            }
        } else {
#pragma unroll
            for (int m = 0; m < 16; ++m) {
                const int ib = m / JB, jb = m % JB;
                mfma_acc(acc[ib][jb], fa[0][ib], fb[0][jb]);
                if (m % 2 == 1) read_frag(1, sA, sB, 1, m / 2);
                if (m % 4 == 3 && more) issue_one(m / 4);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        // mid-chunk barrier: chunk g+1 is complete in LDS for everyone, nobody reads chunk g any more
        wait_mid(more);
        __builtin_amdgcn_s_waitcnt(waitcnt_lgkm0());
        __builtin_amdgcn_sched_barrier(0);
        bare_barrier();
        __builtin_amdgcn_sched_barrier(0);
        // ---------------- step (g, 1): MFMAs from buffer 1, fragments (g+1, 0) into buffer 0 --------------
        const bool next = g + 1 < total;
#pragma unroll
        for (int m = 0; m < 16; ++m) {
            const int ib = m / JB, jb = m % JB;
            mfma_acc(acc[ib][jb], fa[1][ib], fb[1][jb]);
            // buffer 0 is free once the MFMAs of step (g,0) have read it, which they have: they were issued before
            if (m % 2 == 1 && next) read_frag(0, sA1, sB1, 0, m / 2);
            if (m % 4 == 3 && more) issue_one(4 + m / 4);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (more) issue_end();
        sA = sA1;
        sB = sB1;
        if (++c == NC) {
            // the last MFMAs must have written their accumulators before vector instructions read them
            asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15\n\ts_nop 15" ::: "memory");
            epilogue(tile, qb, par);
            c = 0;
            par ^= 1;
            tile += step_tile;
            qb += step_qb;
            if (qb >= nqb) {
                qb -= nqb;
                ++tile;
            }
        }
    }

    if (!SAMPLE && lane == 0) {
        const uint32_t cap = (uint32_t)p.region_cap;
        p.region_cnt[blockIdx.x * NW + wave] = wave_cnt < cap ? wave_cnt : cap;
    }
}

template <class C> hipError_t launch_scan_big_cfg(bool sample, int grid, const ScanArgs &a, hipStream_t s)
{
    static bool attr_done[2] = {false, false};
    auto *fn = sample ? &kb_scan_big_kernel<C, true> : &kb_scan_big_kernel<C, false>;
    if (!attr_done[sample]) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(fn), hipFuncAttributeMaxDynamicSharedMemorySize, C::SMEM_BYTES);
        if (e != hipSuccess) return e;
        attr_done[sample] = true;
    }
    hipLaunchKernelGGL(fn, dim3(grid), dim3(C::THREADS), C::SMEM_BYTES, s, a);
    return hipGetLastError();
}

}  // namespace kbi
