// Kernels of one tree-verification step (paper, section "Custom-Designed Decoding Tree":
// the target LLM checks every node of the draft tree in one pass under tree attention,
// then the longest greedily-accepted path is kept).  Layouts are described in
// fv_device.hpp.  Every kernel checks its own bounds; the host checks shapes first.
#pragma once
#include "fv_device.hpp"
#include "fv_types.hpp"

// ============================================================================ ingest
// Tree ingest: ancestor sets, positions, rotary table.  One block.
// mask[i] = mask[parent[i]] | bit(i), built by walking the parent chain (at most
// depth steps); position of node i = L + depth[i]  (node i continues the sequence
// prefix ++ root path, so it sits depth[i] places after the root at position L).
struct IngestArgs {
    const int32_t* tok_in;   // [3][cap]: tokens, parent, depth
    int cap, T, Tp, L, half_d;
    double log2_base;
    uint64_t* mask;          // [Tp][4]
    int32_t* pos;            // [Tp]
    float2* rope_cs;         // [Tp][half_d]  (cos, sin)
    uint8_t* anc;            // [Tp][FV_CANON_DEPTH + 1]: node i's ancestor at depth d, for nodes no deeper than that (or null)
};

#ifndef FV_TS
#define FV_TS(k)   // tuning aid: a stand-alone timing harness defines this to record a time stamp
#endif
#ifndef FV_PH
#define FV_PH_DECL   // tuning aid: per-phase cycle sums inside a pipeline stage
#define FV_PH(k)
#define FV_PH_END
#endif

static __global__ __launch_bounds__(256) void k_ingest(IngestArgs a) {
    // one workgroup per four rows: their ancestor masks (a short chain of dependent loads each) and
    // their rows of the rotary table (double-precision sincos, one or two entries per thread)
    const int tid = threadIdx.x;
    const int32_t* parent = a.tok_in + a.cap;
    const int32_t* depth = a.tok_in + 2 * a.cap;
    const int t0 = blockIdx.x * 4, t1 = (t0 + 4 < a.Tp) ? t0 + 4 : a.Tp;
    for (int i = t0 + tid; i < t1; i += 256) {
        uint64_t m[4] = {0, 0, 0, 0};
        int p = 0;
        if (i < a.T) {
            int j = i, guard = 0;
            const bool by_depth = a.anc && depth[i] <= FV_CANON_DEPTH;
            while (j >= 0 && guard++ < FV_MAX_TREE) {   // host validated parent[j] < j; guard bounds the walk anyway
                m[j >> 6] |= 1ull << (j & 63);
                if (by_depth && depth[j] >= 0 && depth[j] <= FV_CANON_DEPTH) a.anc[i * (FV_CANON_DEPTH + 1) + depth[j]] = (uint8_t)j;
                j = parent[j];
            }
            p = a.L + depth[i];
        }
        for (int w = 0; w < 4; ++w) a.mask[i * 4 + w] = m[w];
        a.pos[i] = p;
    }
    const int n = t1 * a.half_d;
    for (int e = t0 * a.half_d + tid; e < n; e += 256) {
        const int t = e / a.half_d, i = e % a.half_d;
        const int p = (t < a.T) ? a.L + depth[t] : 0;
        // angle = pos * base^(-2i/d), d = 2*half_d
        const double inv_freq = exp2(-(double)i / (double)a.half_d * a.log2_base);
        double s, c;
        sincos((double)p * inv_freq, &s, &c);
        a.rope_cs[e] = make_float2((float)c, (float)s);
    }
}

// ============================================================================ embed
// x[:, t] = E[tok[t]];  also emits the first GEMM's input  xb = x * gain  (un-normalised;
// the RMSNorm scale 1/sqrt(mean(x^2)+eps) is applied to the GEMM result instead, it is a
// per-token factor) and the per-strip partial sums of squares.
struct EmbedArgs {
    const void* table;       // [V][h]
    const int32_t* tok;      // [cap]
    const float* gain;       // [h]
    float* x;                // [h/4][Tp][4]
    void* xb;                // vector-major [h/E][Tp][E]
    float* ssq_part;         // [h/32][Tp]
    int h, T, Tp;
};

template <typename EL>
__global__ void k_embed(EmbedArgs a) {
    const int s = blockIdx.x, t = threadIdx.x;
    if (t >= a.Tp) return;
    float ssq = 0.f;
    for (int q = 0; q < 8; ++q) {
        const int f0 = s * 32 + q * 4;
        float v[4] = {0.f, 0.f, 0.f, 0.f};
        if (t < a.T) {
            const size_t base = (size_t)a.tok[t] * a.h + f0;
            for (int c = 0; c < 4; ++c) v[c] = Tr<EL>::load(a.table, base + c);
        }
        ((float4*)a.x)[(size_t)(f0 >> 2) * a.Tp + t] = make_float4(v[0], v[1], v[2], v[3]);
        store4_act<EL>(a.xb, a.Tp, f0, t, v[0] * a.gain[f0], v[1] * a.gain[f0 + 1], v[2] * a.gain[f0 + 2],
                       v[3] * a.gain[f0 + 3]);
        ssq += v[0] * v[0] + v[1] * v[1] + v[2] * v[2] + v[3] * v[3];
    }
    a.ssq_part[(size_t)s * a.Tp + t] = ssq;
}

// ============================================================================ skinny GEMM
// Y^T[N, Tp] = W[N, K] * X^T[K, Tp] with T = 16..256 tokens: the weights are streamed
// once from HBM, the activations come from L2 through LDS.  The (row-group x K-batch)
// space is cut into G equal contiguous ranges, one per workgroup (stream-K), so all CUs
// stream the same number of bytes whatever N and K are.  A workgroup is R wavefronts;
// wavefront w owns strip w of the row group and all of them share the X chunk in LDS.
// Each range piece that lies in one row group is a "segment".  A segment that covers the
// whole K range goes straight from registers to the epilogue; otherwise its fp32
// accumulators go to `part`, the workgroup takes a ticket on the row group's counter, and
// the workgroup that draws the last ticket sums all segments of the group in ascending
// workgroup order (so the result does not depend on who arrives last) and runs the epilogue.
enum { EPI_QKV = 0, EPI_RESID = 1, EPI_SWIGLU = 2, EPI_LOGITS = 3 };

// n 32-bit words to zero (a template so that every translation unit may hold it)
template <int UNUSED>
__global__ void k_zero_words(uint32_t* p, size_t n) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}

struct GemmArgs {
    const uint4* Wt;     // tiled weights [NG*R strips][NB][FRAGS][64] x 16 B
    const uint4* X;      // vector-major [NB*16][Tp] x 16 B
    const uint4* zeros;  // 32 KiB of zeros (what the direct kernels' padded stages load)
    float* part;         // partial tiles, fp32: [G][segmax][tiles of the kernel][1024]
    unsigned part_bytes; // size of that area (the 128-bit exchange addresses it through a bounds-checked buffer descriptor)
    int* tickets;        // [NG], zero on entry, left zero on exit (shared-activation kernel; the direct kernels draw no tickets)
    // Direct / paired kernels (fv_gemm_direct.hpp): the partial area is all zeros at the start of a launch and
    // left all zeros; a stored partial value carries `mark` in its lowest mantissa bit (1; 0 only in the host's
    // test of the time-out).  spin_limit: re-reads of a tile that has not arrived before the finishing
    // workgroup gives up, stores 1 to *fault and carries on with what it has.
    unsigned mark, spin_limit;
    unsigned* fault;
    int NG, NB, G, segmax;
    int aligned;         // direct kernels: workgroup ranges end on row-group boundaries (no partial tiles)
    // stream-K split, precomputed on the host: range start of every workgroup (G+1 entries), its
    // first row group, and the first / last contributing workgroup of every row group
    const int* tab_u0; const int* tab_g0; const int* tab_cf; const int* tab_cl;
    // Deferred reduction (shared-activation kernel, 128 / 256 tokens): a segment that does not cover
    // the whole K range only stores its partial tiles, and k_gemm_fix, launched right behind, reduces
    // the n_fix row groups that have several contributors with one wavefront per tile.
    int defer, n_fix;
    const int4* fix_groups;  // [n_fix] row groups with more than one contributor: (group, first and last contributor, the first one's segment index)
    float* rinv_out;         // [Tp] RMSNorm factors handed from k_gemm to k_gemm_fix
    int T, n_strips;     // real tokens; strips that carry real rows
    // RMSNorm statistics of the input (QKV, SWIGLU, LOGITS): rinv[t] = rsqrt(sum_s ssq_in[s][t] / h + eps)
    const float* ssq_in; // [n_ssq][Tp]
    int n_ssq;
    float inv_h, eps;
    // EPI_QKV: rotate q and k, write q (vector-major), k and v into the cache at slot L + t.
    // bf16: q is kept as two bf16 tensors, q_out + q_lo_out (the second holds what the first lost to
    // rounding), so that the scores see q at about 16 mantissa bits: the attention kernel has matrix
    // cycles to spare, and rounding q to one bf16 moved the logits of a 32-layer model as much as the
    // whole K cache's rounding does.
    void* q_out;
    void* q_lo_out;
    void* kcache;        // this layer's K slabs [Hkv][S_pad*D]
    void* vcache;
    const float2* rope_cs;   // [Tp][D/2]
    int Hq, Hkv, L, S_pad;
    // EPI_RESID: x = x_in + y (x_in may be x); xb = x * gain_next; partial sums of squares of the new x
    const float* x_in;
    float* x;
    void* xb;
    const float* gain_next;
    float* ssq_out;      // [n_strips][Tp]
    // EPI_SWIGLU: act = silu(gate) * up
    void* act;
    // EPI_LOGITS
    float* logits;       // [Tp][Vpad]
    int Vpad;
};

// Epilogue of one 32-row strip x 32-token block, in accumulator layout: lane (tl, g), acc[i] is
// row 8*(i/4) + 4*g + i%4 of the strip for token tb*32 + tl.
// Inputs of an epilogue that do not depend on the GEMM result.  A caller that has to wait for
// something else first (the partial-tile exchange) requests them before that wait and hands them in.
//   EPI_RESID: x = the residual rows, gain = the next norm's gains of this lane's 16 outputs
//   EPI_QKV (q and k strips): x[2*pr], x[2*pr+1] = the four (cos, sin) pairs of rotary indices
//              16*j + 8*pr + 4*g .. +3 at this lane's token
struct EpiPre { float4 x[4], gain[4]; };
typedef EpiPre ResidPre;
__device__ __forceinline__ void resid_preload(const GemmArgs& a, int Tp, int strip, int tb, int lane, EpiPre& p) {
    const int t = tb * 32 + (lane & 31), g = lane >> 5;
#pragma unroll
    for (int blk = 0; blk < 4; ++blk) {
        const int f0 = strip * 32 + 8 * blk + 4 * g;
        p.x[blk] = ((const float4*)a.x_in)[(size_t)(f0 >> 2) * Tp + t];
        p.gain[blk] = *(const float4*)(a.gain_next + f0);
    }
}
template <int D>
__device__ __forceinline__ bool rope_preload(const GemmArgs& a, int strip, int tb, int lane, EpiPre& p) {
    constexpr int SPH = D / 32;
    const int t = tb * 32 + (lane & 31), g = lane >> 5, j = strip % SPH;
    if (strip / SPH >= a.Hq + a.Hkv) return false;   // a v strip: no rotation
#pragma unroll
    for (int pr = 0; pr < 2; ++pr) {
        const float4* cp = (const float4*)(a.rope_cs + (size_t)t * (D / 2) + 16 * j + 8 * pr + 4 * g);
        p.x[2 * pr] = cp[0];
        p.x[2 * pr + 1] = cp[1];
    }
    return true;
}

template <typename EL, int D, int EPI>
__device__ __forceinline__ void gemm_epilogue(const GemmArgs& a, int Tp, int strip, int tb, int lane, float (&acc)[16],
                                              const float* rinv_lds, const EpiPre& pre, bool have_pre) {
    const int tl = lane & 31, g = lane >> 5;
    const int t = tb * 32 + tl;
    if constexpr (EPI == EPI_RESID) {
        float ssq = 0.f;
#pragma unroll
        for (int blk = 0; blk < 4; ++blk) {
            const int f0 = strip * 32 + 8 * blk + 4 * g;
            float4 xv = pre.x[blk], gn = pre.gain[blk];
            if (!have_pre) { xv = ((const float4*)a.x_in)[(size_t)(f0 >> 2) * Tp + t]; gn = *(const float4*)(a.gain_next + f0); }
            xv.x += acc[4 * blk]; xv.y += acc[4 * blk + 1]; xv.z += acc[4 * blk + 2]; xv.w += acc[4 * blk + 3];
            st_f4((float4*)a.x + (size_t)(f0 >> 2) * Tp + t, xv);
            store4_act<EL>(a.xb, Tp, f0, t, xv.x * gn.x, xv.y * gn.y, xv.z * gn.z, xv.w * gn.w);
            ssq += xv.x * xv.x + xv.y * xv.y + xv.z * xv.z + xv.w * xv.w;
        }
        ssq += __shfl_xor(ssq, 32);
        if (g == 0) st_f32(a.ssq_out + (size_t)strip * Tp + t, ssq);
    } else {
        const float rs = rinv_lds[t];
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[i] *= rs;
        if constexpr (EPI == EPI_LOGITS) {
#pragma unroll
            for (int blk = 0; blk < 4; ++blk) {
                const int f0 = strip * 32 + 8 * blk + 4 * g;
                st_f4((float4*)(a.logits + (size_t)t * a.Vpad + f0),
                           make_float4(acc[4 * blk], acc[4 * blk + 1], acc[4 * blk + 2], acc[4 * blk + 3]));
            }
        } else if constexpr (EPI == EPI_SWIGLU) {
            // strip covers activation features [16*strip, 16*strip+16): accumulator blocks 0,2 are
            // gate rows, blocks 1,3 the matching up rows
#pragma unroll
            for (int pr = 0; pr < 2; ++pr) {
                float o[4];
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const float gt = acc[8 * pr + c], up = acc[8 * pr + 4 + c];
                    o[c] = gt / (1.f + __expf(-gt)) * up;
                }
                store4_act<EL>(a.act, Tp, 16 * strip + 8 * pr + 4 * g, t, o[0], o[1], o[2], o[3]);
            }
        } else {  // EPI_QKV
            constexpr int SPH = D / 32;   // strips per head
            const int head = strip / SPH, j = strip % SPH;
            if (head < a.Hq + a.Hkv) {
                // q or k head: blocks (0,1) and (2,3) are rotary pairs (i, i + D/2)
                float lo_v[2][4], hi_v[2][4];
#pragma unroll
                for (int pr = 0; pr < 2; ++pr) {
                    // (cos, sin) of indices 16*j + 8*pr + 4*g + c in the first half of the head, c = 0..3
                    float4 c01 = pre.x[2 * pr], c23 = pre.x[2 * pr + 1];
                    if (!have_pre) {
                        const float4* cp = (const float4*)(a.rope_cs + (size_t)t * (D / 2) + 16 * j + 8 * pr + 4 * g);
                        c01 = cp[0]; c23 = cp[1];
                    }
                    const float co[4] = {c01.x, c01.z, c23.x, c23.z}, si[4] = {c01.y, c01.w, c23.y, c23.w};
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const float x1 = acc[8 * pr + c], x2 = acc[8 * pr + 4 + c];
                        lo_v[pr][c] = x1 * co[c] - x2 * si[c];
                        hi_v[pr][c] = x2 * co[c] + x1 * si[c];
                    }
                }
                if (head < a.Hq) {
#pragma unroll
                    for (int pr = 0; pr < 2; ++pr) {
                        const int f1 = head * D + 16 * j + 8 * pr + 4 * g;
                        store4_act<EL>(a.q_out, Tp, f1, t, lo_v[pr][0], lo_v[pr][1], lo_v[pr][2], lo_v[pr][3]);
                        store4_act<EL>(a.q_out, Tp, f1 + D / 2, t, hi_v[pr][0], hi_v[pr][1], hi_v[pr][2], hi_v[pr][3]);
                        if constexpr (Tr<EL>::E == 8) {
                            store4_act<EL>(a.q_lo_out, Tp, f1, t, bf16_residual(lo_v[pr][0]), bf16_residual(lo_v[pr][1]),
                                           bf16_residual(lo_v[pr][2]), bf16_residual(lo_v[pr][3]));
                            store4_act<EL>(a.q_lo_out, Tp, f1 + D / 2, t, bf16_residual(hi_v[pr][0]), bf16_residual(hi_v[pr][1]),
                                           bf16_residual(hi_v[pr][2]), bf16_residual(hi_v[pr][3]));
                        }
                    }
                } else if (t < a.T) {
                    const int kh = head - a.Hq;
                    char* slab = (char*)a.kcache + (size_t)kh * a.S_pad * D * Tr<EL>::ESZ;
                    const int pos = a.L + t;   // cache SLOT of tree node t (its rotary position is L + depth)
                    // four consecutive features of one position are contiguous in the slab (they lie in
                    // one 2E-feature fragment row): one 8- or 16-byte store each
#pragma unroll
                    for (int pr = 0; pr < 2; ++pr) {
                        const int f1 = 16 * j + 8 * pr + 4 * g;
                        st_cache4<EL>(slab, kcache_index<EL, D>(pos, f1), lo_v[pr]);
                        st_cache4<EL>(slab, kcache_index<EL, D>(pos, f1 + D / 2), hi_v[pr]);
                    }
                }
            } else if (t < a.T) {
                const int kh = head - a.Hq - a.Hkv;
                char* slab = (char*)a.vcache + (size_t)kh * a.S_pad * D * Tr<EL>::ESZ;
                const int pos = a.L + t;
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int f = 32 * j + 8 * (i >> 2) + 4 * g + (i & 3);
                    st_elem<EL>(slab, vcache_index<EL, D>(pos, f), acc[i]);
                }
            }
        }
    }
}

template <typename EL, int D, int EPI>
__device__ __forceinline__ void gemm_epilogue(const GemmArgs& a, int Tp, int strip, int tb, int lane, float (&acc)[16],
                                              const float* rinv_lds) {
    EpiPre none;   // never read: have_pre = false
    gemm_epilogue<EL, D, EPI>(a, Tp, strip, tb, lane, acc, rinv_lds, none, false);
}

// One stage of the shared-activation GEMM for one wavefront: FV_FRAGS weight fragments (registers)
// times TB activation tiles each (LDS).  The B tiles of fragment f+1 are requested before the
// MFMAs of fragment f are issued, so an LDS read has TB MFMAs (32 cycles each) to land in;
// between_frags(f) runs after the MFMAs of fragment f have been issued -- the kernel puts a slice
// of the next stages' global loads there, so that the texture-address path works through them
// while the matrix cores are busy instead of after them.
template <typename EL, int TB, typename Between>
__device__ __forceinline__ void gemm_compute(const uint4 (&w)[FV_FRAGS], const uint4* __restrict__ xl,
                                             floatx16 (&acc)[TB], int lane, Between&& between_frags) {
    constexpr int Tp = TB * 32;
    const int t = lane & 31, g = lane >> 5;
    const uint4* xb = xl + g * Tp + t;
    uint4 b[2][TB];
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) b[0][tb] = xb[tb * 32];
#pragma unroll
    for (int f = 0; f < FV_FRAGS; ++f) {
        if (f + 1 < FV_FRAGS) {
#pragma unroll
            for (int tb = 0; tb < TB; ++tb) b[(f + 1) & 1][tb] = xb[2 * (f + 1) * Tp + tb * 32];
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int tb = 0; tb < TB; ++tb) acc[tb] = Tr<EL>::mma(w[f], b[f & 1][tb], acc[tb]);
        __builtin_amdgcn_sched_barrier(0);
        between_frags(f);
        __builtin_amdgcn_sched_barrier(0);
    }
}

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));   // a 16-byte register quad as a first-class value

template <int N, int STRIDE>
__device__ __forceinline__ void ld_vec(uint4 (&dst)[N], const uint4* __restrict__ src) {
#pragma unroll
    for (int v = 0; v < N; ++v) dst[v] = src[v * STRIDE];
}
template <int N, int STRIDE>
__device__ __forceinline__ void ld_x(u32x4 (&dst)[N], const uint4* __restrict__ src) {
#pragma unroll
    for (int v = 0; v < N; ++v) dst[v] = *(const u32x4*)(src + v * STRIDE);
}
template <int N, int STRIDE>
__device__ __forceinline__ void st_lds(uint4* dst, const u32x4 (&src)[N]) {
#pragma unroll
    for (int v = 0; v < N; ++v) *(u32x4*)(dst + v * STRIDE) = src[v];
}
template <int TB>
__device__ __forceinline__ void zero_acc(floatx16 (&acc)[TB]) {
#pragma unroll
    for (int tb = 0; tb < TB; ++tb)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[tb][i] = 0.f;
}

// Ends one segment (a run of K batches of one row group): either straight to the epilogue
// (the segment covered the whole K range) or partials + ticket + last-arriver reduction.
//
// Partial tiles cross XCDs, whose L2s are not coherent with each other, so they are written
// and read with the agent-scope cache policy (write-through stores, loads that do not hit a
// stale line) and no whole-L2 write-back or invalidate is needed.  They move as 128-bit
// accesses (layout per tile [4 register quads][64 lanes][4 floats], 1 KiB per wavefront
// access): a wavefront can have 64 memory operations in flight, and with one-register
// accesses that cap, not the memory system, set the pace of a reduction over many
// contributors.  The 128-bit accesses go through a raw buffer descriptor over the partial
// area, which carries the same policy bit as the agent-scope atomics and bounds-checks
// every address in hardware.
template <typename EL, int TB, int D, int EPI>
__device__ __forceinline__ void gemm_flush(const GemmArgs& a, floatx16 (&acc)[TB], int gi, int seg_batches, int seg,
                                           const float* rinv_lds, int* ticket_lds) {
    constexpr int R = FV_R;
    constexpr int Tp = TB * 32;
    constexpr int TG = TB < 4 ? TB : 4;   // tiles handled together: their loads are in flight at the same time
    // early epilogue inputs; not for the rotary epilogue at 256 tokens, where their registers are spilled
    constexpr bool PRE = (EPI == EPI_RESID || (EPI == EPI_QKV && TB <= 4));
    constexpr int SC1 = 16;               // cache-policy operand of the buffer accesses: agent scope
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int strip = gi * R + wave;
    // what the epilogues of tiles t0 .. t0+TG-1 read besides the GEMM result, requested early
    auto preload = [&](int t0, EpiPre (&pre)[TG]) -> bool {
        bool have = false;
        if constexpr (EPI == EPI_RESID) {
#pragma unroll
            for (int tb = 0; tb < TG; ++tb) resid_preload(a, Tp, strip, t0 + tb, lane, pre[tb]);
            have = true;
        } else if constexpr (EPI == EPI_QKV) {
#pragma unroll
            for (int tb = 0; tb < TG; ++tb) have = rope_preload<D>(a, strip, t0 + tb, lane, pre[tb]);
        }
        return have;
    };
    if (seg_batches == a.NB) {
        // the whole K range of this row group was ours: no partials, no ticket
        if (strip < a.n_strips) {
#pragma unroll
            for (int t0 = 0; t0 < TB; t0 += TG) {
                EpiPre pre[TG];
                const bool have = PRE && preload(t0, pre);
#pragma unroll
                for (int tb = 0; tb < TG; ++tb) {
                    float r[16];
#pragma unroll
                    for (int i = 0; i < 16; ++i) r[i] = acc[t0 + tb][i];
                    gemm_epilogue<EL, D, EPI>(a, Tp, strip, t0 + tb, lane, r, rinv_lds, pre[tb], have);
                }
            }
        }
        return;
    }
    const __amdgpu_buffer_rsrc_t prs = __builtin_amdgcn_make_buffer_rsrc((void*)a.part, 0, (int)a.part_bytes, 0x00020000);   // raw, 32-bit data format
    auto tile_ofs = [&](int wg, int sg, int tb) -> unsigned {   // byte offset of this lane's first quad of a tile
        return ((unsigned)(((wg * a.segmax + sg) * R + wave) * TB + tb) * 1024u + (unsigned)lane * 4u) * 4u;
    };
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) {
        const unsigned o = tile_ofs((int)blockIdx.x, seg, tb);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            u32x4 v;
            v.x = __float_as_uint(acc[tb][4 * q]); v.y = __float_as_uint(acc[tb][4 * q + 1]);
            v.z = __float_as_uint(acc[tb][4 * q + 2]); v.w = __float_as_uint(acc[tb][4 * q + 3]);
            __builtin_amdgcn_raw_buffer_store_b128(v, prs, o + q * 1024u, 0, SC1);
        }
    }
    if (a.defer) return;   // reduced by k_gemm_fix after this launch (the launch boundary orders the two)
    // contributors of row group gi: workgroups c_first..c_last (each has a non-empty range); the
    // ranges are contiguous, so every contributor but the first starts inside the group (its
    // segment index for it is 0)
    const int c_first = a.tab_cf[gi], c_last = a.tab_cl[gi];
    const int seg_first = gi - a.tab_g0[c_first];
    // Release: the payload was stored write-through, so it is enough that every lane's stores
    // have been acknowledged (vmcnt(0): on this target stores count in vmcnt) before the
    // ticket is drawn.
    handoff_release();
    FV_TS(3)
    __syncthreads();
    if (tid == 0)
        *ticket_lds = __hip_atomic_fetch_add(&a.tickets[gi], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    handoff_acquire();
    FV_TS(4)
    const bool last = (*ticket_lds == c_last - c_first);
    if (last) {
        // every other contributor's ticket, hence its acknowledged stores, precede ours
        if (tid == 0) __hip_atomic_store(&a.tickets[gi], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // for the next launch
        if (strip < a.n_strips) {
            // KC contributors x TG tiles (up to 32 KiB per wavefront) are in flight at a time; the
            // sum runs in ascending contributor order, so it does not depend on who arrived last
            constexpr int KC = TG <= 2 ? 4 : (TB <= 4 ? 2 : 1);   // at 256 tokens the activation staging registers leave room for one
#pragma unroll
            for (int t0 = 0; t0 < TB; t0 += TG) {
                EpiPre pre[TG];
                const bool have = PRE && preload(t0, pre);
                float r[TG][16];
#pragma unroll
                for (int tb = 0; tb < TG; ++tb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) r[tb][i] = 0.f;
                for (int c0 = c_first; c0 <= c_last; c0 += KC) {
                    u32x4 v[KC][TG][4];
#pragma unroll
                    for (int k = 0; k < KC; ++k) {
                        const int c = (c0 + k <= c_last) ? c0 + k : c_last;
                        const unsigned o = tile_ofs(c, (c == c_first) ? seg_first : 0, t0);
#pragma unroll
                        for (int tb = 0; tb < TG; ++tb)
#pragma unroll
                            for (int q = 0; q < 4; ++q)
                                v[k][tb][q] = __builtin_amdgcn_raw_buffer_load_b128(prs, o + (tb * 4 + q) * 1024u, 0, SC1);
                    }
#pragma unroll
                    for (int k = 0; k < KC; ++k) {
                        const float m = (c0 + k <= c_last) ? 1.f : 0.f;
#pragma unroll
                        for (int tb = 0; tb < TG; ++tb)
#pragma unroll
                            for (int q = 0; q < 4; ++q) {
                                r[tb][4 * q] += m * __uint_as_float(v[k][tb][q].x);
                                r[tb][4 * q + 1] += m * __uint_as_float(v[k][tb][q].y);
                                r[tb][4 * q + 2] += m * __uint_as_float(v[k][tb][q].z);
                                r[tb][4 * q + 3] += m * __uint_as_float(v[k][tb][q].w);
                            }
                    }
                }
                if (t0 == 0) { FV_TS(5) }
#pragma unroll
                for (int tb = 0; tb < TG; ++tb) gemm_epilogue<EL, D, EPI>(a, Tp, strip, t0 + tb, lane, r[tb], rinv_lds, pre[tb], have);
            }
            FV_TS(6)
        }
    }
    __syncthreads();   // ticket_lds is reused by the next segment
}

template <typename EL, int TB, int D, int EPI>
__global__ __launch_bounds__(64 * FV_R, 1) void k_gemm(GemmArgs a) {
    extern __shared__ uint4 lds[];
    constexpr int R = FV_R;
    constexpr int Tp = TB * 32;
    constexpr int CV = Tp * 16;          // uint4 per X chunk (Tp tokens x 256 B)
    constexpr int XV = CV / (64 * R);    // uint4 per thread per chunk
    static_assert(CV % (64 * R) == 0, "chunk must divide over the workgroup");
    __shared__ float rinv_lds[Tp];
    __shared__ __attribute__((aligned(16))) float red_lds[(EPI == EPI_RESID) ? 4 : 1024];
    __shared__ int ticket_lds;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    if ((int)blockIdx.x >= a.G) return;
    FV_TS(0)

    // This workgroup's units [u0, u1) of the (row group, K batch) space are one software-pipelined
    // stream: the weight tiles and the activation chunk of stage k+2 are requested while stage k is
    // multiplied (weights into the third register set, the chunk into staging registers that go to
    // the other LDS buffer one stage later), across row-group boundaries too.  Every segment (the
    // part of the range inside one row group) is padded to whole rounds of three stages; a padded
    // stage loads zeros as its activation chunk (and one weight line, finite), so the loop body has
    // no conditional, the accumulators stay in the accumulation registers, and the number of loads
    // per stage -- which the wait counts are computed from -- is fixed.
    const long long U = (long long)a.NG * a.NB;   // computed, not looked up: no extra round trip before the first load
    const int u0 = (int)(U * blockIdx.x / a.G);
    const int u1 = (int)(U * (blockIdx.x + 1) / a.G);
    const int g0 = u0 / a.NB;
    int nseg = 1;
    for (int e_ = (g0 + 1) * a.NB; e_ < u1; e_ += a.NB) ++nseg;
    auto segment = [&](int sgm, int& gi, int& b0, int& nb) {
        gi = g0 + sgm;
        b0 = (sgm == 0) ? u0 - g0 * a.NB : 0;
        const int rem = u1 - gi * a.NB;
        nb = (rem < a.NB ? rem : a.NB) - b0;
    };
    // weights are tiled [strip pair][half K batch][2 strips][4 frags]: this wavefront's strip is strip (wave % 2) of pair
    // gi * 2 + wave / 2; a K batch of it is two 4 KiB pieces 8 KiB apart, and batches follow each other 16 KiB apart
    const uint4* __restrict__ wbase = a.Wt + ((size_t)(wave >> 1) * (2 * a.NB) * 2 + (wave & 1)) * (4 * 64) + lane;
    const size_t group_stride = (size_t)R * a.NB * (FV_FRAGS * 64);
    const uint4* const zeros = a.zeros;

    // request position: segment rs, padded stage rj of rn3 (rn real ones), this thread's addresses
    int rs = 0, rj = 0, rn = 0, rn3 = 0;
    const uint4* wp = a.Wt;
    const uint4* xp = zeros;
    auto enter = [&](int sgm) {
        rs = sgm; rj = 0; rn = 0; rn3 = 0; wp = a.Wt; xp = zeros;
        if (rs < nseg) {
            int gi, b0, nb;
            segment(rs, gi, b0, nb);
            rn = nb; rn3 = (nb + 2) / 3 * 3;
            wp = wbase + (size_t)gi * group_stride + (size_t)b0 * (2 * FV_FRAGS * 64);
            xp = a.X + (size_t)b0 * CV + tid;
        }
    };
    auto advance = [&]() {
        ++rj; wp += 2 * FV_FRAGS * 64; xp += CV;
        if (rj >= rn3) enter(rs + 1);
    };
    auto load_w = [&](uint4 (&dst)[FV_FRAGS]) {
        const bool live = rj < rn;
        const uint4* pw = live ? wp : a.Wt;
        const int st = live ? 64 : 0;
#pragma unroll
        for (int f = 0; f < FV_FRAGS; ++f) dst[f] = pw[(f < 4 ? f : f + 4) * st];
    };
    auto load_x = [&](u32x4 (&dst)[XV]) {
        const bool live = rj < rn;
        const uint4* px = live ? xp : zeros;
        const int st = live ? 64 * R : 0;
#pragma unroll
        for (int v = 0; v < XV; ++v) dst[v] = *(const u32x4*)(px + v * st);
    };
    uint4 w[3][FV_FRAGS];
    u32x4 xr[XV];
    enter(0);
    // prologue: W(0) first, so that it is in flight during the statistics below
    load_w(w[0]);
    if constexpr (EPI != EPI_RESID) {
        // RMSNorm factor of every token, while the first weight tiles are in flight.  The
        // [n_ssq][Tp] partial sums of squares are read as float4 (4 tokens) with eight
        // independent loads in flight per thread, then reduced over strip slices in LDS.
        constexpr int C4 = Tp / 4;            // float4 columns
        constexpr int SL = 256 / C4;          // strip slices
        const int col = tid % C4, sl = tid / C4;
        const float4* sp = (const float4*)a.ssq_in + col;
        float4 s4 = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int i0 = sl; i0 < a.n_ssq; i0 += 8 * SL) {
            float4 v[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const int i = i0 + k * SL;
                v[k] = (i < a.n_ssq) ? sp[(size_t)i * C4] : make_float4(0.f, 0.f, 0.f, 0.f);
            }
#pragma unroll
            for (int k = 0; k < 8; ++k) { s4.x += v[k].x; s4.y += v[k].y; s4.z += v[k].z; s4.w += v[k].w; }
        }
        ((float4*)red_lds)[sl * C4 + col] = s4;
        __syncthreads();
        if (tid < Tp) {
            float tot = 0.f;
#pragma unroll
            for (int p = 0; p < SL; ++p) tot += red_lds[p * Tp + tid];
            const float rv = rsqrtf(tot * a.inv_h + a.eps);
            rinv_lds[tid] = rv;
            if (a.defer && blockIdx.x == 0) a.rinv_out[tid] = rv;
        }
    }
    // X(0) -> LDS[0]; then X(1) and W(1) are issued in the same order as inside the loop
    // (activation chunk before weight tiles), so the loop's wait counts hold from the first stage
    load_x(xr);
    st_lds<XV, 64 * R>(lds + tid, xr);
    __builtin_amdgcn_sched_barrier(0);
    advance();   // stage 1
    load_x(xr);
    __builtin_amdgcn_sched_barrier(0);
    load_w(w[1]);
    __builtin_amdgcn_sched_barrier(0);
    __syncthreads();
    FV_TS(1)

    FV_PH_DECL
    int par = 0;   // LDS buffer that holds the current stage's chunk
    // One pipeline stage with weight register set S; the loads it issues (stage + 2) go to set S2.
    // The chunk of stage + 1 goes from its staging registers to the other LDS buffer first (every
    // wavefront is past the barrier, so nobody reads that buffer any more); that frees the staging
    // registers, and the NLD loads of stage + 2 (activation chunk first, then weight tiles) are
    // issued in slices between the fragments of this stage's multiplication.
    constexpr int NLD = XV + FV_FRAGS;
#define FV_STAGE(S, S2)                                                                                 \
    {                                                                                                   \
        st_lds<XV, 64 * R>(lds + (par ^ 1) * CV + tid, xr);                                             \
        __builtin_amdgcn_sched_barrier(0);                                                              \
        FV_PH(1)                                                                                        \
        advance();                                                                                      \
        const bool live_ = rj < rn;                                                                     \
        const uint4* const px_ = live_ ? xp : zeros;                                                    \
        const uint4* const pw_ = live_ ? wp : a.Wt;                                                     \
        const int sx_ = live_ ? 64 * R : 0, sw_ = live_ ? 64 : 0;                                       \
        gemm_compute<EL, TB>(w[S], lds + par * CV, acc, lane, [&](int f) {                              \
            _Pragma("unroll") for (int i_ = f * NLD / FV_FRAGS; i_ < (f + 1) * NLD / FV_FRAGS; ++i_) {  \
                if (i_ < XV) xr[i_] = *(const u32x4*)(px_ + i_ * sx_);                                  \
                else w[S2][i_ - XV] = pw_[((i_ - XV) < 4 ? (i_ - XV) : (i_ - XV) + 4) * sw_];                                             \
            }                                                                                           \
        });                                                                                             \
        FV_PH(0)                                                                                        \
        __syncthreads();                                                                                \
        FV_PH(3)                                                                                        \
        par ^= 1;                                                                                       \
    }

    for (int sgm = 0; sgm < nseg; ++sgm) {
        int gi, b0, nb;
        segment(sgm, gi, b0, nb);
        const int rounds = (nb + 2) / 3;
        floatx16 acc[TB];
        zero_acc<TB>(acc);
        for (int r = 0; r < rounds; ++r) {
            FV_STAGE(0, 2)
            FV_STAGE(1, 0)
            FV_STAGE(2, 1)
        }
        FV_TS(2)
        gemm_flush<EL, TB, D, EPI>(a, acc, gi, nb, sgm, rinv_lds, &ticket_lds);
    }
    FV_TS(7)
    FV_PH_END
#undef FV_STAGE
}

// Second half of a deferred reduction: one wavefront per (row group with several contributors,
// strip, token block) tile sums the contributors' partial tiles in ascending workgroup order and
// runs the epilogue.  Spreading the tiles over the whole chip instead of leaving each row group
// to its last arriver matters at 128 / 256 tokens, where a row group's partials are 0.5-1 MiB and
// one CU pulls them in at ~60 GB/s.
template <typename EL, int TB, int D, int EPI>
__global__ __launch_bounds__(256) void k_gemm_fix(GemmArgs a) {
    constexpr int R = FV_R;
    constexpr int Tp = TB * 32;
    constexpr int SC1 = 16;
    __shared__ float rinv_lds[Tp];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    if constexpr (EPI != EPI_RESID) {
        if (tid < Tp) rinv_lds[tid] = a.rinv_out[tid];
        __syncthreads();
    }
    const int tile = blockIdx.x * 4 + wave;
    if (tile >= a.n_fix * R * TB) return;
    const int4 rec = a.fix_groups[tile / (R * TB)];   // one load: nothing else stands between kernel entry and the partial loads
    const int gi = rec.x, c_first = rec.y, c_last = rec.z, seg_first = rec.w;
    const int r = (tile / TB) % R, tb = tile % TB;
    const int strip = gi * R + r;
    if (strip >= a.n_strips) return;
    EpiPre pre;
    bool have = false;
    if constexpr (EPI == EPI_RESID) { resid_preload(a, Tp, strip, tb, lane, pre); have = true; }
    if constexpr (EPI == EPI_QKV) have = rope_preload<D>(a, strip, tb, lane, pre);
    const __amdgpu_buffer_rsrc_t prs = __builtin_amdgcn_make_buffer_rsrc((void*)a.part, 0, (int)a.part_bytes, 0x00020000);
    float acc[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0.f;
    for (int c0 = c_first; c0 <= c_last; c0 += 4) {   // four contributors in flight, summed in ascending order
        u32x4 v[4][4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int c = (c0 + k <= c_last) ? c0 + k : c_last;
            const unsigned o = ((unsigned)(((c * a.segmax + ((c == c_first) ? seg_first : 0)) * R + r) * TB + tb) * 1024u + (unsigned)lane * 4u) * 4u;
#pragma unroll
            for (int q = 0; q < 4; ++q) v[k][q] = __builtin_amdgcn_raw_buffer_load_b128(prs, o + q * 1024u, 0, SC1);
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const float m = (c0 + k <= c_last) ? 1.f : 0.f;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                acc[4 * q] += m * __uint_as_float(v[k][q].x);
                acc[4 * q + 1] += m * __uint_as_float(v[k][q].y);
                acc[4 * q + 2] += m * __uint_as_float(v[k][q].z);
                acc[4 * q + 3] += m * __uint_as_float(v[k][q].w);
            }
        }
    }
    gemm_epilogue<EL, D, EPI>(a, Tp, strip, tb, lane, acc, rinv_lds, pre, have);
}

#include "fv_gemm_direct.hpp"

// ============================================================================ tree attention
// For node t and query head qh: softmax over {cache slots 0..L-1} U {tree slots L+j : j in
// ancestors-or-self(t)} of q.k/sqrt(D), times V.  A workgroup handles one (query head,
// block of 32 nodes); its four wavefronts take every fourth 32-key block, keep online-softmax
// statistics, and are merged through LDS.  Scores are computed transposed (keys x nodes)
// so that each lane owns one node: the node's 256-bit ancestor set sits in registers and
// is tested per key, and the probabilities are already in B-operand order for V^T * P^T.
struct AttnArgs {
    const uint4* q;          // vector-major [Hq*D/E][Tp]
    const uint4* q_lo;       // bf16 only: the part of q that q's bf16 rounding lost (same layout)
    const uint4* kc;         // this layer's K slabs
    const uint4* vc;
    void* out;               // vector-major [Hq*D/E][Tp]
    const uint64_t* mask;    // [Tp][4]
    int Tp, T, L, Hq, Hkv, S_pad;
    int TK;                  // step rows whose keys exist, slots L .. L+TK-1 (= T in a verification step; a drafting pass also sees
                             // the rows of the phase's earlier passes); the masks have no bits at or above TK
    float scale;
    // key split: every (head, node block) item is shared by `ks` workgroups, each taking a
    // contiguous run of 32-key blocks; their (max, sum, unnormalised output) triples meet in
    // `part` ([item*ks + k][D/32 * 1024 + 64] floats) behind one ticket per item
    int ks;
    float* part;
    int* tickets;
};

#define FV_ATTN_SMEM_FLOATS(D) (3 * ((D) / 32) * 64 * 16 + 8 * 32 + 4)
#define FV_ATTN_PART_FLOATS(D) (((D) / 32) * 1024 + 64)

// One (query head, block of 32 nodes) item, key part `part` of a.ks.
template <typename EL, int D>
__device__ __forceinline__ void attn_body(const AttnArgs& a, int item, int part, float* smem) {
    constexpr int E = Tr<EL>::E;
    constexpr int NF = D / (2 * E);      // K frags per key block
    constexpr int NQ = 32 / (2 * E);     // V frags per (key block, 32 features)
    constexpr int DB = D / 32;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int tl = lane & 31, g = lane >> 5;
    const int TB = a.Tp >> 5;
    const int qh = item / TB, tb = item % TB;
    const int kh = qh / (a.Hq / a.Hkv);
    const int t = tb * 32 + tl;

    constexpr bool SPLIT = (E == 8);   // bf16: q and the probabilities enter the matrix cores as hi + lo pairs
    uint4 qf[NF], qfl[SPLIT ? NF : 1];
#pragma unroll
    for (int fr = 0; fr < NF; ++fr) qf[fr] = a.q[((size_t)(qh * (D / E) + 2 * fr + g)) * a.Tp + t];
    if constexpr (SPLIT) {
#pragma unroll
        for (int fr = 0; fr < NF; ++fr) qfl[fr] = a.q_lo[((size_t)(qh * (D / E) + 2 * fr + g)) * a.Tp + t];
    }
    uint64_t mk[4];
#pragma unroll
    for (int w = 0; w < 4; ++w) mk[w] = (t < a.T) ? a.mask[t * 4 + w] : 0ull;

    const size_t slab_vecs = (size_t)a.S_pad * D / E;
    const uint4* kslab = a.kc + (size_t)kh * slab_vecs;
    const uint4* vslab = a.vc + (size_t)kh * slab_vecs;

    floatx16 o[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[db][i] = 0.f;
    float m_run = -1e30f, l_run = 0.f;

    const int n_keys = a.L + a.TK;
    const int nkb = (n_keys + 31) >> 5;
    const int kb_lo = nkb * part / a.ks, kb_hi = nkb * (part + 1) / a.ks;   // this workgroup's key blocks
    const int lidx = tl * 2 + g;   // position of this lane's 16 bytes inside a 1 KiB tile
    // all K and V tiles of a block are requested before the first is used: one memory round trip
    // per block instead of two
    auto load_block = [&](uint4 (&kt)[NF], uint4 (&vt)[DB * NQ], int kb) {
        const uint4* kp = kslab + (size_t)kb * NF * 64 + lidx;
        const uint4* vp = vslab + (size_t)kb * DB * NQ * 64 + lidx;
#pragma unroll
        for (int fr = 0; fr < NF; ++fr) kt[fr] = kp[fr * 64];
#pragma unroll
        for (int j = 0; j < DB * NQ; ++j) vt[j] = vp[j * 64];
    };
    auto use_block = [&](const uint4 (&kt)[NF], const uint4 (&vt)[DB * NQ], int kb) {
        // two accumulation chains (a dependent MFMA waits ~50 cycles for its predecessor, two
        // interleaved chains issue back to back), added at the end
        floatx16 s, s1;
#pragma unroll
        for (int i = 0; i < 16; ++i) { s[i] = 0.f; s1[i] = 0.f; }
#pragma unroll
        for (int fr = 0; fr < NF; fr += 2) {
            s = Tr<EL>::mma(kt[fr], qf[fr], s);
            s1 = Tr<EL>::mma(kt[fr + 1], qf[fr + 1], s1);
            if constexpr (SPLIT) {
                s = Tr<EL>::mma(kt[fr], qfl[fr], s);
                s1 = Tr<EL>::mma(kt[fr + 1], qfl[fr + 1], s1);
            }
        }
#pragma unroll
        for (int i = 0; i < 16; ++i) s[i] += s1[i];

        // Visibility of the block's 32 keys for this lane's node as one 32-bit word (bit j: key
        // kb*32 + j): prefix keys are visible to every node, a tree key n only if bit n of the node's
        // ancestor mask is set (the mask has no bits at or above T).  The block's offset into the
        // tree, n0, is the same for the whole wavefront, so the window is cut out of the 256-bit
        // mask with uniform shifts and no per-element branch.
        uint32_t vbits = 0xffffffffu;
        const int n0 = kb * 32 - a.L;   // tree index of the block's first key
        if (n0 > -32) {
            uint32_t win;
            if (n0 < 0) {
                win = ((1u << (-n0)) - 1u) | ((uint32_t)mk[0] << (-n0));
            } else {
                const int w = n0 >> 6, sh = n0 & 63;
                const uint64_t lo = (w == 0) ? mk[0] : (w == 1) ? mk[1] : (w == 2) ? mk[2] : (w == 3) ? mk[3] : 0ull;
                const uint64_t hi = (w == 0) ? mk[1] : (w == 1) ? mk[2] : (w == 2) ? mk[3] : 0ull;
                win = (uint32_t)(sh ? ((lo >> sh) | (hi << (64 - sh))) : lo);
            }
            vbits = win >> (4 * g);
        }
        float p[16];
        float mx = -1e30f;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const bool vis = (vbits >> (8 * (i >> 2) + (i & 3))) & 1u;   // key 8*(i/4) + 4*g + i%4 of the block
            p[i] = vis ? s[i] * a.scale : -1e30f;
            mx = fmaxf(mx, p[i]);
        }
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        // Lazy rescale: the running reference m_run only has to be near the running maximum, not equal
        // to it -- exp(score - m_run) stays below e^8 as long as no row's maximum has grown by more than
        // 8 since the reference was set, which fp32 sums and bf16 probabilities hold without loss.  The
        // accumulators (64 registers, a read-multiply-write each) are rescaled only when some row of the
        // wavefront crosses that bound; after the first blocks of a long key range that is rare.
        const float m_cand = fmaxf(m_run, mx);
        if (__any(m_cand - m_run > 8.f)) {
            const float alpha = __expf(m_run - m_cand);
            l_run *= alpha;
            m_run = m_cand;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int i = 0; i < 16; ++i) o[db][i] *= alpha;
        }
        float psum = 0.f;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            p[i] = (p[i] > -1e29f) ? __expf(p[i] - m_run) : 0.f;
            psum += p[i];
        }
        l_run += psum;
        uint4 pb[NQ], pbl[SPLIT ? NQ : 1];
#pragma unroll
        for (int q = 0; q < NQ; ++q) pb[q] = Tr<EL>::pack(p + q * E);
        if constexpr (SPLIT) {   // what the probabilities lose to bf16 rounding goes through the matrix cores too
#pragma unroll
            for (int i = 0; i < 16; ++i) p[i] = bf16_residual(p[i]);
#pragma unroll
            for (int q = 0; q < NQ; ++q) pbl[q] = Tr<EL>::pack(p + q * E);
        }
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int q = 0; q < NQ; ++q) {
                o[db] = Tr<EL>::mma(vt[db * NQ + q], pb[q], o[db]);
                if constexpr (SPLIT) o[db] = Tr<EL>::mma(vt[db * NQ + q], pbl[q], o[db]);
            }
    };
    for (int kb = kb_lo + wave; kb < kb_hi; kb += 4) {
        uint4 kt[NF], vt[DB * NQ];
        load_block(kt, vt, kb);
        __builtin_amdgcn_sched_barrier(0);   // the 16 requests stay together, ahead of everything that uses them
        use_block(kt, vt, kb);
    }
    l_run += __shfl_xor(l_run, 32);

    // ---- merge the four wavefronts: 1..3 park their accumulators in LDS, wavefront 0 combines
    float* so = smem;                              // [3][DB][64][16]
    float* sm = smem + 3 * DB * 64 * 16;           // [4][32] running max
    float* sl = sm + 4 * 32;                       // [4][32] running sum
    if (wave > 0) {
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int q = 0; q < 4; ++q)
                ((float4*)so)[(((wave - 1) * DB + db) * 64 + lane) * 4 + q] =
                    make_float4(o[db][4 * q], o[db][4 * q + 1], o[db][4 * q + 2], o[db][4 * q + 3]);
    }
    if (g == 0) { sm[wave * 32 + tl] = m_run; sl[wave * 32 + tl] = l_run; }
    __syncthreads();
    int* ticket_lds = (int*)(sl + 4 * 32);
    float M = -1e30f, lsum = 0.f;
    float r[DB][16];
    if (wave == 0) {
#pragma unroll
        for (int w = 0; w < 4; ++w) M = fmaxf(M, sm[w * 32 + tl]);
        float wgt[4];
#pragma unroll
        for (int w = 0; w < 4; ++w) { wgt[w] = __expf(sm[w * 32 + tl] - M); lsum += wgt[w] * sl[w * 32 + tl]; }
#pragma unroll
        for (int db = 0; db < DB; ++db) {
#pragma unroll
            for (int i = 0; i < 16; ++i) r[db][i] = wgt[0] * o[db][i];
#pragma unroll
            for (int w = 1; w < 4; ++w)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const float4 v = ((const float4*)so)[(((w - 1) * DB + db) * 64 + lane) * 4 + q];
                    r[db][4 * q] += wgt[w] * v.x; r[db][4 * q + 1] += wgt[w] * v.y;
                    r[db][4 * q + 2] += wgt[w] * v.z; r[db][4 * q + 3] += wgt[w] * v.w;
                }
        }
    }
    if (a.ks == 1) {
        if (wave == 0) {
            const float inv = (lsum > 0.f) ? 1.f / lsum : 0.f;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int blk = 0; blk < 4; ++blk)
                    store4_act<EL>(a.out, a.Tp, qh * D + db * 32 + 8 * blk + 4 * g, t, r[db][4 * blk] * inv,
                                        r[db][4 * blk + 1] * inv, r[db][4 * blk + 2] * inv, r[db][4 * blk + 3] * inv);
        }
        return;
    }
    // ---- several workgroups share this item: partial triple out (agent-scope atomic stores,
    // acknowledged), ticket, and the last arriver combines all parts in part order
    constexpr int PF = FV_ATTN_PART_FLOATS(D);
    if (wave == 0) {
        float* pp = a.part + (size_t)(item * a.ks + part) * PF + lane;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int i = 0; i < 16; ++i) __hip_atomic_store(pp + (db * 16 + i) * 64, r[db][i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (g == 0) {
            __hip_atomic_store(pp + DB * 1024, M, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);         // lanes 0..31
            __hip_atomic_store(pp + DB * 1024 + 32, lsum, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        handoff_release();
        if (lane == 0) *ticket_lds = __hip_atomic_fetch_add(&a.tickets[item], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    handoff_acquire();
    if (*ticket_lds != a.ks - 1) return;
    if (tid == 0) __hip_atomic_store(&a.tickets[item], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // for the next use
    // wavefront w combines 32-feature block w (blocks beyond D/32 have no wavefront).  Everything it
    // needs from the up to eight parts is requested in one go (parts beyond ks re-read part 0 and
    // get weight zero), so the merge costs one memory round trip.
    const float* base = a.part + (size_t)item * a.ks * PF;
    for (int db = wave; db < DB; db += 4) {
        float mc[8], lc[8], v[8][16];
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            const float* cp = base + (size_t)(c < a.ks ? c : 0) * PF;
            mc[c] = __hip_atomic_load(cp + DB * 1024 + tl, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            lc[c] = __hip_atomic_load(cp + DB * 1024 + 32 + tl, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
            for (int i = 0; i < 16; ++i) v[c][i] = __hip_atomic_load(cp + (db * 16 + i) * 64 + lane, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        float Mx = -1e30f;
#pragma unroll
        for (int c = 0; c < 8; ++c) if (c < a.ks) Mx = fmaxf(Mx, mc[c]);
        float accv[16], ltot = 0.f;
#pragma unroll
        for (int i = 0; i < 16; ++i) accv[i] = 0.f;
#pragma unroll
        for (int c = 0; c < 8; ++c) {   // part order
            const float wc = (c < a.ks) ? __expf(mc[c] - Mx) : 0.f;
            ltot += wc * lc[c];
#pragma unroll
            for (int i = 0; i < 16; ++i) accv[i] += wc * v[c][i];
        }
        const float inv = (ltot > 0.f) ? 1.f / ltot : 0.f;
#pragma unroll
        for (int blk = 0; blk < 4; ++blk)
            store4_act<EL>(a.out, a.Tp, qh * D + db * 32 + 8 * blk + 4 * g, t, accv[4 * blk] * inv, accv[4 * blk + 1] * inv,
                                accv[4 * blk + 2] * inv, accv[4 * blk + 3] * inv);
    }
}

// grid = items * ks
template <typename EL, int D>
__global__ __launch_bounds__(256) void k_attn(AttnArgs a) {
    __shared__ __attribute__((aligned(16))) float smem[FV_ATTN_SMEM_FLOATS(D)];
    // Workgroups go to the 8 XCDs round-robin (workgroup b runs on XCD b % 8) and every XCD has its
    // own L2, so all node blocks and key parts of a query head -- and the query heads that share a
    // KV head -- are given to workgroups of one XCD: a head's K/V then comes from HBM once and is
    // re-read from that L2, instead of once per XCD that touches it.  (Only locality depends on the
    // dispatch order; any other order computes the same thing.)
    int item = blockIdx.x / a.ks, part = blockIdx.x % a.ks;
    if ((a.Hq & 7) == 0) {
        const int x = blockIdx.x & 7, j = blockIdx.x >> 3;
        const int TB = a.Tp >> 5, per_head = TB * a.ks;
        const int head = x * (a.Hq >> 3) + j / per_head, w = j % per_head;
        item = head * TB + w / a.ks;
        part = w % a.ks;
    }
    attn_body<EL, D>(a, item, part, smem);
}

#include "fv_attn_canon.hpp"

// ============================================================================ argmax
// Greedy choice per node: wavefront shuffle reduction on (value, index), lowest index on ties.
// A row that holds a NaN or an infinity has no greedy choice: its entry becomes -1, which the
// scan turns into an error for the whole step.
struct ArgmaxArgs {
    const float* logits;   // [Tp][Vpad]
    int32_t* am;           // [Tp]
    int V, Vpad;
};

__device__ __forceinline__ void argmax_combine(float& v, int& i, float ov, int oi) {
    if (ov > v || (ov == v && oi < i)) { v = ov; i = oi; }
}

static __global__ __launch_bounds__(256) void k_argmax(ArgmaxArgs a) {
    __shared__ float sv[4];
    __shared__ int si[4];
    __shared__ int sbad[4];
    const int t = blockIdx.x, tid = threadIdx.x;
    const float* row = a.logits + (size_t)t * a.Vpad;
    float bv = -INFINITY;
    int bi = 0x7fffffff;
    bool bad = false;
    // eight 16-byte loads in flight per thread (the row is a latency chain otherwise: one load per
    // trip of a loop the compiler does not pipeline); indices past Vpad are not touched, values
    // between V and Vpad are skipped
    for (int v0 = tid * 4; v0 < a.V; v0 += 8 * 256 * 4) {
        float4 x[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int v = v0 + k * 256 * 4;
            x[k] = (v < a.V) ? *(const float4*)(row + v) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int v = v0 + k * 256 * 4;
            const float xs[4] = {x[k].x, x[k].y, x[k].z, x[k].w};
#pragma unroll
            for (int c = 0; c < 4; ++c)
                if (v + c < a.V) {
                    // finite <=> |x| < inf; false for NaN too
                    bad = bad || !(__builtin_fabsf(xs[c]) < INFINITY);
                    argmax_combine(bv, bi, xs[c], v + c);
                }
        }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const float ov = __shfl_xor(bv, off);
        const int oi = __shfl_xor(bi, off);
        argmax_combine(bv, bi, ov, oi);
    }
    const bool wbad = __any(bad);
    if ((tid & 63) == 0) { sv[tid >> 6] = bv; si[tid >> 6] = bi; sbad[tid >> 6] = wbad ? 1 : 0; }
    __syncthreads();
    if (tid == 0) {
        for (int w = 1; w < 4; ++w) argmax_combine(bv, bi, sv[w], si[w]);
        a.am[t] = (sbad[0] | sbad[1] | sbad[2] | sbad[3]) ? -1 : bi;
    }
}

// ============================================================================ longest accepted path
// Single block.  match[i] = (i is the root) or tok[i] == argmax[parent[i]]; node i is
// accepted iff every node of its ancestor set matches; best = deepest accepted node, lowest
// index among equals; path = members of best's ancestor set in increasing index (= depth) order.
// Features of the accepted path for the next drafting round: row j = the LM head's input (final
// RMSNorm of the last layer's output) of path node j, j = 0..accepted_len, fp32 [max_tree][h].
// One block per possible path position; blocks beyond the path leave at once.
struct FeatureArgs {
    const FvResult* res;
    const float* x;          // residual stream after the last layer, fp32 [h/4][Tp][4]
    const float* ssq;        // its per-strip sums of squares [h/32][Tp]
    const float* gain;       // final norm gain [h]
    float* out;              // [max_tree][h]
    int h, Tp;
    float inv_h, eps;
};

static __global__ __launch_bounds__(256) void k_features(FeatureArgs a) {
    __shared__ float red[256];
    const int j = blockIdx.x, tid = threadIdx.x;
    if (j > a.res->accepted_len) return;
    const int t = a.res->path[j];
    float s = 0.f;
    for (int i = tid; i < a.h / 32; i += 256) s += a.ssq[(size_t)i * a.Tp + t];
    red[tid] = s;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if (tid < w) red[tid] += red[tid + w];
        __syncthreads();
    }
    const float rinv = rsqrtf(red[0] * a.inv_h + a.eps);
    for (int f = tid; f < a.h; f += 256)
        a.out[(size_t)j * a.h + f] = a.x[((size_t)(f >> 2) * a.Tp + t) * 4 + (f & 3)] * rinv * a.gain[f];
}

struct ScanArgs {
    const int32_t* tok_in;   // [3][cap]
    int cap, T;
    const uint64_t* mask;
    const int32_t* am;
    FvResult* res;
};

static __global__ __launch_bounds__(256) void k_scan(ScanArgs a) {
    __shared__ unsigned long long mbits[4];
    __shared__ int best_key;
    __shared__ int any_bad;
    const int i = threadIdx.x;
    const int32_t* tok = a.tok_in;
    const int32_t* parent = a.tok_in + a.cap;
    const int32_t* depth = a.tok_in + 2 * a.cap;
    if (i < 4) mbits[i] = 0ull;
    if (i == 0) { best_key = -1; any_bad = 0; }
    __syncthreads();
    if (i < a.T && a.am[i] < 0) any_bad = 1;   // a row without a greedy choice (non-finite logits)
    if (i < a.T) {
        const bool match = (i == 0) || (tok[i] == a.am[parent[i]]);
        if (match) atomicOr(&mbits[i >> 6], 1ull << (i & 63));
    }
    __syncthreads();
    if (i < a.T) {
        bool ok = true;
        for (int w = 0; w < 4; ++w) ok = ok && ((a.mask[i * 4 + w] & ~mbits[w]) == 0ull);
        if (ok) atomicMax(&best_key, depth[i] * 512 + (511 - i));
    }
    __syncthreads();
    if (any_bad) {   // no decision: accepted_len = FV_SCAN_NONFINITE tells the host, nothing is compacted
        if (i == 0) { a.res->accepted_len = FV_SCAN_NONFINITE; a.res->next_token = -1; a.res->best = 0; a.res->pad = 0; }
        return;
    }
    const int best = 511 - (best_key & 511);
    if (i == 0) {
        a.res->accepted_len = depth[best];
        a.res->next_token = a.am[best];
        a.res->best = best;
        a.res->pad = 0;
    }
    if (i < a.T) {
        const uint64_t* mb = a.mask + best * 4;
        if ((mb[i >> 6] >> (i & 63)) & 1ull) {
            int rank = 0;
            for (int w = 0; w < (i >> 6); ++w) rank += __popcll(mb[w]);
            rank += __popcll(mb[i >> 6] & ((1ull << (i & 63)) - 1ull));
            a.res->path[rank] = i;
            if (rank >= 1) a.res->accepted_tokens[rank - 1] = tok[i];
        }
    }
}

// ============================================================================ non-greedy acceptance
// Multi-step speculative sampling over the tree (the non-greedy setting of the paper's Appendix
// "Tree Structure"; verification in the SpecInfer manner, section "Custom-Designed Decoding Tree").
// Single block.  Starting at the root with w = exp((logits[node] - max) / temperature): the children of
// the current node are tried in index order; child c with token x is accepted iff
// u_accept[c] * q[x] * sum(w) <= w[x]; on rejection w becomes the positive part of w - sum(w) * q and the
// next child is tried against it.  q is row `node` of draft_probs, or a point mass on x if draft_probs
// is null (then rejection just strikes x from w).  When no child is accepted the next token is the first
// v with cumsum(w)[v] > u_sample[node] * sum(w).  All of it in fp64 (the decisions are thresholds on sums
// of 32000 terms; fp64 keeps both sides of a comparison with a CPU implementation within ~1e-13 of each
// other), in a fixed order, so the result is reproducible.
struct SampledArgs {
    const int32_t* tok_in;     // [3][cap]: tokens, parent, depth
    int cap, T;
    const float* logits;       // [Tp][Vpad]
    int V, Vpad;
    double inv_temperature;
    const float* draft_probs;  // [T][V] or null
    const double* u_accept;    // [T]
    const double* u_sample;    // [T]
    double* work;              // [Vpad]
    FvResult* res;
};

#define FV_SAMPLED_THREADS 1024

// sum of one value per thread over the block, in a fixed order; every thread gets the result
__device__ __forceinline__ double block_sum_f64(double v, double* red) {
    const int tid = threadIdx.x;
    red[tid] = v;
    __syncthreads();
    for (int w = FV_SAMPLED_THREADS / 2; w > 0; w >>= 1) {
        if (tid < w) red[tid] += red[tid + w];
        __syncthreads();
    }
    const double r = red[0];
    __syncthreads();
    return r;
}

static __global__ __launch_bounds__(FV_SAMPLED_THREADS) void k_accept_sampled(SampledArgs a) {
    __shared__ double red[FV_SAMPLED_THREADS];
    __shared__ int s_flag, s_pick;
    __shared__ float s_maxf[FV_SAMPLED_THREADS / 64];
    const int tid = threadIdx.x;
    const int32_t* tok = a.tok_in;
    const int32_t* parent = a.tok_in + a.cap;
    const int chunk = (a.V + FV_SAMPLED_THREADS - 1) / FV_SAMPLED_THREADS;   // contiguous tokens per thread
    const int v0 = tid * chunk, v1 = (v0 + chunk < a.V) ? v0 + chunk : a.V;
    int cur = 0, len = 0, next_token = -1;
    bool bad = false;
    if (tid == 0) a.res->path[0] = 0;
    for (int hop = 0; hop < a.T && next_token < 0 && !bad; ++hop) {
        const float* row = a.logits + (size_t)cur * a.Vpad;
        // ---- w = exp((row - max) / temperature), S = sum(w)
        float mx = -INFINITY;
        bool nf = false;
        for (int v = v0; v < v1; ++v) { const float x = row[v]; nf = nf || !(__builtin_fabsf(x) < INFINITY); mx = fmaxf(mx, x); }
        for (int off = 32; off >= 1; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
        if (tid == 0) s_flag = 0;
        __syncthreads();
        if (nf) s_flag = 1;
        if ((tid & 63) == 0) s_maxf[tid >> 6] = mx;
        __syncthreads();
        if (s_flag) { bad = true; break; }
        for (int k = 0; k < FV_SAMPLED_THREADS / 64; ++k) mx = fmaxf(mx, s_maxf[k]);
        const double zmax = (double)mx * a.inv_temperature;
        auto fill = [&]() {
            double ls = 0.0;
            for (int v = v0; v < v1; ++v) { const double w = exp((double)row[v] * a.inv_temperature - zmax); a.work[v] = w; ls += w; }
            return ls;
        };
        double S = block_sum_f64(fill(), red);
        // ---- the children of cur, in index order
        int taken = -1;
        for (int c = cur + 1; c < a.T && taken < 0; ++c) {
            if (parent[c] != cur) continue;            // uniform: every thread reads the same value
            const int x = tok[c];
            const double qx = a.draft_probs ? (double)a.draft_probs[(size_t)cur * a.V + x] : 1.0;
            __syncthreads();                            // a.work[x] as left by the previous child's update
            const double lhs = a.u_accept[c] * qx * S, rhs = a.work[x];
            if (lhs <= rhs) { taken = c; break; }
            __syncthreads();                            // everyone has read work[x] before it changes
            double ls = 0.0;
            if (a.draft_probs) {
                const float* q = a.draft_probs + (size_t)cur * a.V;
                for (int v = v0; v < v1; ++v) { const double w = fmax(a.work[v] - S * (double)q[v], 0.0); a.work[v] = w; ls += w; }
            } else {
                for (int v = v0; v < v1; ++v) { if (v == x) a.work[v] = 0.0; ls += a.work[v]; }
            }
            double S2 = block_sum_f64(ls, red);
            if (!(S2 > 0.0)) S2 = block_sum_f64(fill(), red);   // nothing left besides what was rejected (probability zero): keep the last p
            S = S2;
        }
        if (taken >= 0) {
            ++len;
            if (tid == 0) { a.res->path[len] = taken; a.res->accepted_tokens[len - 1] = tok[taken]; }
            cur = taken;
            continue;
        }
        // ---- draw: the first v with cumsum(w)[v] > target
        __syncthreads();
        const double target = a.u_sample[cur] * S;
        double ls = 0.0;
        for (int v = v0; v < v1; ++v) ls += a.work[v];
        // inclusive prefix over the threads' chunk sums (fixed order)
        red[tid] = ls;
        __syncthreads();
        for (int off = 1; off < FV_SAMPLED_THREADS; off <<= 1) {
            const double add = (tid >= off) ? red[tid - off] : 0.0;
            __syncthreads();
            red[tid] += add;
            __syncthreads();
        }
        const double before = red[tid] - ls;
        if (tid == 0) s_pick = 0x7fffffff;
        __syncthreads();
        if (ls > 0.0 && before <= target && target < red[tid]) {
            double c = before;
            int pick = -1;
            for (int v = v0; v < v1; ++v) { c += a.work[v]; if (c > target) { pick = v; break; } }
            if (pick < 0) for (int v = v1 - 1; v >= v0; --v) if (a.work[v] > 0.0) { pick = v; break; }   // rounding inside the chunk
            if (pick >= 0) atomicMin(&s_pick, pick);
        }
        __syncthreads();
        if (s_pick == 0x7fffffff) {
            // target at or beyond the total (u_sample ~ 1 and rounding): the last token that has any mass
            for (int v = v1 - 1; v >= v0; --v) if (a.work[v] > 0.0) { atomicMax(&s_flag, v + 1); break; }
            __syncthreads();
            next_token = s_flag - 1;
        } else {
            next_token = s_pick;
        }
    }
    if (tid == 0) {
        if (bad || next_token < 0) { a.res->accepted_len = FV_SCAN_NONFINITE; a.res->next_token = -1; a.res->best = 0; }
        else { a.res->accepted_len = len; a.res->next_token = next_token; a.res->best = cur; }
        a.res->pad = 0;
    }
}

// ============================================================================ KV compaction
// For every layer and KV head: cache slot L + j <- cache slot L + path[j], j = 0..a.
// Tree K/V were written at slots L + node index; path[j] >= j, and thread e moves element e
// for j = 0, 1, ... in order, so a slot is always read before it can be overwritten.
struct CompactArgs {
    void* kcache;      // [NL][Hkv][S_pad*D]
    void* vcache;
    const FvResult* res;
    int L, S_pad;
};

template <typename EL, int D>
__global__ void k_compact(CompactArgs a) {
    const int e = threadIdx.x;   // feature, blockDim.x == D
    char* ks = (char*)a.kcache + (size_t)blockIdx.x * a.S_pad * D * Tr<EL>::ESZ;
    char* vs = (char*)a.vcache + (size_t)blockIdx.x * a.S_pad * D * Tr<EL>::ESZ;
    typedef typename Tr<EL>::elem_t el_t;
    const int n = a.res->accepted_len;
    for (int j = 0; j <= n && j < FV_MAX_TREE; ++j) {
        const int src = a.res->path[j];
        if (src == j) continue;
        ((el_t*)ks)[kcache_index<EL, D>(a.L + j, e)] = ((el_t*)ks)[kcache_index<EL, D>(a.L + src, e)];
        ((el_t*)vs)[vcache_index<EL, D>(a.L + j, e)] = ((el_t*)vs)[vcache_index<EL, D>(a.L + src, e)];
    }
}

// ============================================================================ helpers: weight tiling, KV read-back
struct TileArgs {
    const void* src0; const void* src1; const void* src2;
    uint4* out;
    int kind, n_strips_pad, NB, K, N;
    int Hq, Hkv, D, F;
};

template <typename EL>
__global__ __launch_bounds__(256) void k_tile(TileArgs a) {
    constexpr int E = Tr<EL>::E;
    const size_t total = (size_t)a.n_strips_pad * a.NB * FV_FRAGS * 64;
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const int lane = idx & 63;
    // output order [strip pair][half K batch][strip of the pair][4 frags][64 lanes]
    const size_t tile = idx >> 6;
    const int ff = (int)(tile & 3), r = (int)((tile >> 2) & 1);
    const size_t pj = tile >> 3;
    const int j = (int)(pj % ((size_t)2 * a.NB));
    const int strip = 2 * (int)(pj / ((size_t)2 * a.NB)) + r;
    const int frag = 4 * j + ff;
    const int m = lane & 31, g = lane >> 5;
    const int k0 = frag * 2 * E + g * E;
    const void* src = nullptr;
    long long row = -1;
    if (a.kind == TILE_NAT) {
        row = (long long)strip * 32 + m;
        src = a.src0;
        if (row >= a.N) row = -1;
    } else if (a.kind == TILE_QKV) {
        const int sph = a.D / 32, head = strip / sph, j = strip % sph;
        const int blk = m >> 3, within = m & 7;
        const int paired = (blk & 1) * (a.D / 2) + 16 * j + (blk >> 1) * 8 + within;
        if (head < a.Hq) { src = a.src0; row = (long long)head * a.D + paired; }
        else if (head < a.Hq + a.Hkv) { src = a.src1; row = (long long)(head - a.Hq) * a.D + paired; }
        else if (head < a.Hq + 2 * a.Hkv) { src = a.src2; row = (long long)(head - a.Hq - a.Hkv) * a.D + 32 * j + m; }
    } else {
        const int blk = m >> 3;
        const int f = 16 * strip + (blk >> 1) * 8 + (m & 7);
        if (f < a.F) { row = f; src = (blk & 1) ? a.src1 : a.src0; }
    }
    uint4 v = make_uint4(0, 0, 0, 0);
    if (row >= 0 && k0 < a.K)   // K is a multiple of E, so a vector is all inside or all outside
        v = *(const uint4*)((const char*)src + ((size_t)row * a.K + k0) * Tr<EL>::ESZ);
    a.out[idx] = v;
}

struct ReadKvArgs {
    const void* kcache; const void* vcache;   // this layer's slabs
    float* k_out; float* v_out;               // [n][Hkv][D]
    int slot0, n, Hkv, S_pad;
};
template <typename EL, int D>
__global__ void k_read_kv(ReadKvArgs a) {
    const int e = threadIdx.x, kh = blockIdx.y, j = blockIdx.x;
    if (j >= a.n) return;
    const char* ks = (const char*)a.kcache + (size_t)kh * a.S_pad * D * Tr<EL>::ESZ;
    const char* vs = (const char*)a.vcache + (size_t)kh * a.S_pad * D * Tr<EL>::ESZ;
    const size_t o = ((size_t)j * a.Hkv + kh) * D + e;
    a.k_out[o] = Tr<EL>::load(ks, kcache_index<EL, D>(a.slot0 + j, e));
    a.v_out[o] = Tr<EL>::load(vs, vcache_index<EL, D>(a.slot0 + j, e));
}
