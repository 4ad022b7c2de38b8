// Tile configurations of the scan kernel: X(id, key dtype, TK, TQ, WM, WN, RBA, NSTAGE, WGPC)
//   TK x TQ      keys x queries per work item         WM x WN  wavefront grid inside the workgroup
//   RBA          bytes of each key row per d-chunk    NSTAGE   chunk buffers in LDS
//   WGPC         workgroups resident per compute unit (LDS and registers are budgeted for it)
// (12, 16: small tiles for knowledge bases of some ten thousand rows, where a query is bound by the latency of its
//  launches and more, shorter work items finish sooner)
#pragma once
#define KB_SCAN_CONFIGS_BF16(X)                  \
    X(1, KB_BF16, 128, 32, 4, 1, 128, 3, 2)      \
    X(2, KB_BF16, 128, 128, 2, 2, 64, 4, 2)      \
    X(3, KB_BF16, 128, 256, 2, 2, 64, 3, 2)      \
    X(12, KB_BF16, 64, 64, 2, 2, 128, 4, 2)      \
    X(16, KB_BF16, 64, 128, 2, 2, 128, 3, 2)
#define KB_SCAN_CONFIGS_F32(X)                   \
    X(1, KB_F32, 128, 32, 4, 1, 128, 3, 2)       \
    X(2, KB_F32, 128, 128, 2, 2, 64, 4, 2)       \
    X(3, KB_F32, 128, 256, 2, 2, 64, 3, 2)
#define KB_SCAN_CONFIGS_FP8(X)                   \
    X(1, KB_FP8_E4M3, 128, 32, 4, 1, 64, 3, 2)   \
    X(2, KB_FP8_E4M3, 128, 128, 2, 2, 64, 3, 2)  \
    X(3, KB_FP8_E4M3, 128, 256, 2, 2, 64, 3, 1)
// ... with fp8 queries as well (key type KB_FP8_Q8 inside the kernels): every row length, every batch size
#define KB_SCAN_CONFIGS_FP8_Q8(X)                \
    X(6, KB_FP8_Q8, 128, 64, 2, 2, 64, 3, 2)     \
    X(7, KB_FP8_Q8, 128, 128, 2, 2, 64, 3, 2)    \
    X(8, KB_FP8_Q8, 128, 256, 2, 2, 64, 3, 1)

// Software-pipelined configurations (kb_scan_sp.hpp): XS(id, key dtype, TQ, NSA, NSB); 256-row tiles, 512 threads,
// NSA / NSB = ring depth of key / query chunks in LDS.
// bf16: the loads are issued between the MFMAs (IL mode)
#define KB_SCAN_SP_CONFIGS_BF16_IL(XI) \
    XI(17, KB_BF16, 256, 5, 4)
#define KB_SCAN_SP_CONFIGS_FP8(XS)  \
    XS(4, KB_FP8_E4M3, 256, 3, 3)
// ... with fp8 queries as well (the fp8 matrix instruction): XQ(id, key dtype, TQ, NSA, NSB)
#define KB_SCAN_SP_CONFIGS_FP8_Q8(XQ) \
    XQ(5, KB_FP8_E4M3, 256, 5, 4)

// Full-line configurations (kb_scan_wide.hpp): XW(id, key dtype, TQ); 256-row tiles, 512 threads, 128-byte row pieces.
#define KB_SCAN_WIDE_CONFIGS_BF16(XW) \
    XW(18, KB_BF16, 256)              \
    XW(19, KB_BF16, 128)
// ... for fp8 keys with fp8 queries
#define KB_SCAN_WIDE_CONFIGS_FP8_Q8(XW) \
    XW(20, KB_FP8_E4M3, 256)
