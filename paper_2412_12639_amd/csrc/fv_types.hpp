// Constants and the result record shared by the kernels and the host side.
#pragma once
#include <stdint.h>

#define FV_MAX_TREE 256
#define FV_R 4            // strips (wavefronts) per GEMM workgroup
#define FV_FRAGS 8        // weight frags per K batch

#define FV_DRAFT_KMAX 8   // largest k of the semi-autoregressive drafter
#define FV_DRAFT_MMAX 32  // longest top list per drafter row

#define FV_SCAN_NONFINITE (-2)   // FvResult.accepted_len when some node's logits hold a NaN or an infinity

// Result of the longest-accepted-path scan, written by the device and copied to the host.
struct FvResult {
    int32_t accepted_len, next_token, best, pad;
    int32_t path[FV_MAX_TREE];
    int32_t accepted_tokens[FV_MAX_TREE];
};

enum { TILE_NAT = 0, TILE_QKV = 1, TILE_GU = 2 };   // weight re-tiling: natural row order, q|k|v with rotary pairing, gate/up interleaved
