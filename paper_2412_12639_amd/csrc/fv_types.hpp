// Constants and the result record shared by the kernels and the host side.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#define FV_MAX_TREE 256
#define FV_CANON_DEPTH 32 // deepest node that the step-independent form of the attention takes (see fv_attn_canon.hpp)
#define FV_R 4            // strips (wavefronts) per GEMM workgroup
#define FV_FRAGS 8        // weight frags per K batch

#define FV_DRAFT_KMAX 8   // largest k of the semi-autoregressive drafter
#define FV_DRAFT_MMAX 32  // longest top list per drafter row

#define FV_SCAN_NONFINITE (-2)   // FvResult.accepted_len when some node's logits hold a NaN or an infinity

// Result of the longest-accepted-path scan, written by the device and copied to the host.
struct FvResult {
    int32_t accepted_len, next_token, best, pad;
    uint32_t fault, pad2[3];   // fault: set by a GEMM whose partial-tile wait ran out (never cleared: the context is unusable then)
    int32_t path[FV_MAX_TREE];
    int32_t accepted_tokens[FV_MAX_TREE];
};

enum { TILE_NAT = 0, TILE_QKV = 1, TILE_GU = 2 };   // weight re-tiling: natural row order, q|k|v with rotary pairing, gate/up interleaved

// Far-key parts of the step-independent attention (fv_attn_canon.hpp): fixed absolute positions.
// Part j holds 4 * canon_part_run(j) blocks of 32 keys starting at block canon_part_b0(j).
#define FV_CANON_MAX_PARTS 24  // far parts a step may have (positions up to 15872)

__host__ __device__ inline int canon_part_run(int j) { return j < 4 ? 1 : j < 8 ? 2 : j < 12 ? 4 : 8; }   // blocks per wavefront
__host__ __device__ inline int canon_part_b0(int j) {
    return j < 4 ? 4 * j : j < 8 ? 16 + 8 * (j - 4) : j < 12 ? 48 + 16 * (j - 8) : 112 + 32 * (j - 12);
}
__host__ __device__ inline int canon_parts(int nfb) {   // parts that hold blocks [0, nfb)
    int j = 0;
    while (canon_part_b0(j) < nfb) ++j;
    return j;
}

