// Kernels of one tree-verification step (paper, section "Custom-Designed Decoding Tree":
// the target LLM checks every node of the draft tree in one pass under tree attention,
// then the longest greedily-accepted path is kept).  Layouts are described in
// fv_device.hpp.  Every kernel checks its own bounds; the host checks shapes first.
#pragma once
#include "fv_device.hpp"

#define FV_MAX_TREE 256
#define FV_R 4            // strips (wavefronts) per GEMM workgroup
#define FV_FRAGS 8        // weight frags per K batch

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
};

__global__ __launch_bounds__(256) void k_ingest(IngestArgs a) {
    const int tid = threadIdx.x;
    const int32_t* parent = a.tok_in + a.cap;
    const int32_t* depth = a.tok_in + 2 * a.cap;
    for (int i = tid; i < a.Tp; i += 256) {
        uint64_t m[4] = {0, 0, 0, 0};
        int p = 0;
        if (i < a.T) {
            int j = i, guard = 0;
            while (j >= 0 && guard++ < FV_MAX_TREE) {   // host validated parent[j] < j; guard bounds the walk anyway
                m[j >> 6] |= 1ull << (j & 63);
                j = parent[j];
            }
            p = a.L + depth[i];
        }
        for (int w = 0; w < 4; ++w) a.mask[i * 4 + w] = m[w];
        a.pos[i] = p;
    }
    const int n = a.Tp * a.half_d;
    for (int e = tid; e < n; e += 256) {
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
// Each range piece that lies in one row group is a "segment" whose fp32 accumulators go
// to `part`; k_fixup sums the segments of a row group in a fixed order (deterministic)
// and applies the epilogue.
struct GemmArgs {
    const uint4* Wt;     // tiled weights [NG*R strips][NB][FRAGS][64] x 16 B
    const uint4* X;      // vector-major [NB*16][Tp] x 16 B
    float* part;         // [G][segmax][R][TB][64][16] fp32
    int NG, NB, G, segmax;
    // side job of workgroup 0: finish the RMSNorm statistics of the input
    const float* ssq_part;   // [n_ssq][Tp] or null
    float* rinv;             // [Tp]
    int n_ssq;
    float inv_h, eps;
};

template <typename EL, int TB>
__device__ __forceinline__ void gemm_compute(const uint4 (&w)[FV_FRAGS], const uint4* __restrict__ xl,
                                             floatx16 (&acc)[TB], int lane) {
    constexpr int Tp = TB * 32;
    const int t = lane & 31, g = lane >> 5;
#pragma unroll
    for (int f = 0; f < FV_FRAGS; ++f) {
#pragma unroll
        for (int tb = 0; tb < TB; ++tb) {
            const uint4 b = xl[(2 * f + g) * Tp + tb * 32 + t];
            acc[tb] = Tr<EL>::mma(w[f], b, acc[tb]);
        }
    }
}

template <typename EL, int TB>
__global__ __launch_bounds__(64 * FV_R, 1) void k_gemm(GemmArgs a) {
    extern __shared__ uint4 lds[];
    constexpr int R = FV_R;
    constexpr int Tp = TB * 32;
    constexpr int CV = Tp * 16;          // uint4 per X chunk (Tp tokens x 256 B)
    constexpr int XV = CV / (64 * R);    // uint4 per thread per chunk
    static_assert(CV % (64 * R) == 0, "chunk must divide over the workgroup");
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;

    if (blockIdx.x == 0 && a.ssq_part != nullptr) {
        for (int t = tid; t < Tp; t += 64 * R) {
            float s = 0.f;
            for (int i = 0; i < a.n_ssq; ++i) s += a.ssq_part[(size_t)i * Tp + t];
            a.rinv[t] = rsqrtf(s * a.inv_h + a.eps);
        }
    }
    if ((int)blockIdx.x >= a.G) return;

    const long long U = (long long)a.NG * a.NB;
    long long u0 = U * blockIdx.x / a.G;
    const long long u1 = U * (blockIdx.x + 1) / a.G;
    int seg = 0;
    while (u0 < u1) {
        const int gi = (int)(u0 / a.NB);
        const int b0 = (int)(u0 - (long long)gi * a.NB);
        const int nb = (int)((u1 - u0 < (long long)(a.NB - b0)) ? (u1 - u0) : (long long)(a.NB - b0));

        floatx16 acc[TB];
#pragma unroll
        for (int tb = 0; tb < TB; ++tb)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[tb][i] = 0.f;

        const uint4* __restrict__ wp = a.Wt + ((size_t)(gi * R + wave) * a.NB + b0) * (FV_FRAGS * 64) + lane;
        const uint4* __restrict__ xp = a.X + (size_t)b0 * CV + tid;
        uint4 w0[FV_FRAGS], w1[FV_FRAGS], xr[XV];
#pragma unroll
        for (int f = 0; f < FV_FRAGS; ++f) w0[f] = wp[f * 64];
#pragma unroll
        for (int v = 0; v < XV; ++v) xr[v] = xp[v * 64 * R];
#pragma unroll
        for (int v = 0; v < XV; ++v) lds[tid + v * 64 * R] = xr[v];
        __syncthreads();

        for (int b = 0; b < nb; b += 2) {
            // the next X chunk is always fetched (the last one twice: it is an L2 hit) so that
            // its staging registers are written and read unconditionally
            const bool has1 = b + 1 < nb;
            const int bx1 = has1 ? b + 1 : b;
#pragma unroll
            for (int v = 0; v < XV; ++v) xr[v] = xp[(size_t)bx1 * CV + v * 64 * R];
            if (has1) {
#pragma unroll
                for (int f = 0; f < FV_FRAGS; ++f) w1[f] = wp[(size_t)(b + 1) * (FV_FRAGS * 64) + f * 64];
            }
            gemm_compute<EL, TB>(w0, lds, acc, lane);
#pragma unroll
            for (int v = 0; v < XV; ++v) lds[CV + tid + v * 64 * R] = xr[v];
            __syncthreads();
            if (!has1) break;
            const bool has2 = b + 2 < nb;
            const int bx2 = has2 ? b + 2 : b + 1;
#pragma unroll
            for (int v = 0; v < XV; ++v) xr[v] = xp[(size_t)bx2 * CV + v * 64 * R];
            if (has2) {
#pragma unroll
                for (int f = 0; f < FV_FRAGS; ++f) w0[f] = wp[(size_t)(b + 2) * (FV_FRAGS * 64) + f * 64];
            }
            gemm_compute<EL, TB>(w1, lds + CV, acc, lane);
#pragma unroll
            for (int v = 0; v < XV; ++v) lds[tid + v * 64 * R] = xr[v];
            __syncthreads();
        }

        float4* pp = (float4*)a.part + ((((size_t)blockIdx.x * a.segmax + seg) * R + wave) * TB) * (64 * 4) + lane * 4;
#pragma unroll
        for (int tb = 0; tb < TB; ++tb)
#pragma unroll
            for (int q = 0; q < 4; ++q)
                pp[tb * 64 * 4 + q] = make_float4(acc[tb][4 * q], acc[tb][4 * q + 1], acc[tb][4 * q + 2], acc[tb][4 * q + 3]);
        ++seg;
        u0 += nb;
    }
}

// ============================================================================ fix-up + epilogues
enum { EPI_QKV = 0, EPI_RESID = 1, EPI_SWIGLU = 2, EPI_LOGITS = 3 };

struct FixArgs {
    const float* part;
    int NG, NB, G, segmax;
    int Tp, T, n_strips;       // n_strips = strips that carry real rows
    const float* rinv;         // [Tp] RMSNorm factor of the GEMM input (QKV, SWIGLU, LOGITS)
    // EPI_QKV: rotate q and k at pos = L + depth, write q (vector-major), k and v into the cache at slot L + t
    void* q_out;
    void* kcache;              // this layer's K slabs [Hkv][S_pad*D]
    void* vcache;
    const float2* rope_cs;     // [Tp][D/2]
    int Hq, Hkv, L, S_pad;
    // EPI_RESID: x += y; xb = x * gain_next; partial sums of squares of the new x
    float* x;
    void* xb;
    const float* gain_next;
    float* ssq_part;
    // EPI_SWIGLU: act = silu(gate) * up
    void* act;
    // EPI_LOGITS
    float* logits;             // [Tp][Vpad]
    int Vpad;
};

template <typename EL, int D, int EPI>
__global__ __launch_bounds__(256) void k_fixup(FixArgs a) {
    constexpr int R = FV_R;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int TB = a.Tp >> 5;
    const int id = blockIdx.x * 4 + wave;
    const int strip = id / TB, tb = id % TB;
    if (strip >= a.n_strips) return;
    const int gi = strip / R, r = strip % R;

    // ---- sum the segments of row group gi, in ascending workgroup order
    const long long U = (long long)a.NG * a.NB;
    const long long lo = (long long)gi * a.NB, hi = lo + a.NB;
    int wg = (int)(lo * a.G / U);
    while (wg < a.G && U * (wg + 1) / a.G <= lo) ++wg;
    float acc[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0.f;
    for (; wg < a.G; ++wg) {
        const long long w0 = U * wg / a.G, w1 = U * (wg + 1) / a.G;
        if (w0 >= hi) break;
        if (w0 == w1) continue;
        const int seg = gi - (int)(w0 / a.NB);
        const float4* pp = (const float4*)a.part + ((((size_t)wg * a.segmax + seg) * R + r) * TB + tb) * (64 * 4) + lane * 4;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float4 v = pp[q];
            acc[4 * q] += v.x; acc[4 * q + 1] += v.y; acc[4 * q + 2] += v.z; acc[4 * q + 3] += v.w;
        }
    }

    const int tl = lane & 31, g = lane >> 5;
    const int t = tb * 32 + tl;

    if constexpr (EPI == EPI_RESID) {
        float ssq = 0.f;
#pragma unroll
        for (int blk = 0; blk < 4; ++blk) {
            const int f0 = strip * 32 + 8 * blk + 4 * g;
            float4* xp = (float4*)a.x + (size_t)(f0 >> 2) * a.Tp + t;
            float4 xv = *xp;
            xv.x += acc[4 * blk]; xv.y += acc[4 * blk + 1]; xv.z += acc[4 * blk + 2]; xv.w += acc[4 * blk + 3];
            *xp = xv;
            store4_act<EL>(a.xb, a.Tp, f0, t, xv.x * a.gain_next[f0], xv.y * a.gain_next[f0 + 1],
                           xv.z * a.gain_next[f0 + 2], xv.w * a.gain_next[f0 + 3]);
            ssq += xv.x * xv.x + xv.y * xv.y + xv.z * xv.z + xv.w * xv.w;
        }
        ssq += __shfl_xor(ssq, 32);
        if (g == 0) a.ssq_part[(size_t)strip * a.Tp + t] = ssq;
    } else {
        const float rs = a.rinv[t];
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[i] *= rs;
        if constexpr (EPI == EPI_LOGITS) {
#pragma unroll
            for (int blk = 0; blk < 4; ++blk) {
                const int f0 = strip * 32 + 8 * blk + 4 * g;
                *(float4*)(a.logits + (size_t)t * a.Vpad + f0) =
                    make_float4(acc[4 * blk], acc[4 * blk + 1], acc[4 * blk + 2], acc[4 * blk + 3]);
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
                store4_act<EL>(a.act, a.Tp, 16 * strip + 8 * pr + 4 * g, t, o[0], o[1], o[2], o[3]);
            }
        } else {  // EPI_QKV
            constexpr int SPH = D / 32;   // strips per head
            const int head = strip / SPH, j = strip % SPH;
            if (head < a.Hq + a.Hkv) {
                // q or k head: blocks (0,1) and (2,3) are rotary pairs (i, i + D/2)
                float lo_v[2][4], hi_v[2][4];
#pragma unroll
                for (int pr = 0; pr < 2; ++pr)
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const int i1 = 16 * j + 8 * pr + 4 * g + c;     // index in the first half of the head
                        const float2 cs = a.rope_cs[(size_t)t * (D / 2) + i1];
                        const float x1 = acc[8 * pr + c], x2 = acc[8 * pr + 4 + c];
                        lo_v[pr][c] = x1 * cs.x - x2 * cs.y;
                        hi_v[pr][c] = x2 * cs.x + x1 * cs.y;
                    }
                if (head < a.Hq) {
#pragma unroll
                    for (int pr = 0; pr < 2; ++pr) {
                        const int f1 = head * D + 16 * j + 8 * pr + 4 * g;
                        store4_act<EL>(a.q_out, a.Tp, f1, t, lo_v[pr][0], lo_v[pr][1], lo_v[pr][2], lo_v[pr][3]);
                        store4_act<EL>(a.q_out, a.Tp, f1 + D / 2, t, hi_v[pr][0], hi_v[pr][1], hi_v[pr][2], hi_v[pr][3]);
                    }
                } else if (t < a.T) {
                    const int kh = head - a.Hq;
                    char* slab = (char*)a.kcache + (size_t)kh * a.S_pad * D * Tr<EL>::ESZ;
                    const int pos = a.L + t;   // cache SLOT of tree node t (its rotary position is L + depth)
#pragma unroll
                    for (int pr = 0; pr < 2; ++pr)
#pragma unroll
                        for (int c = 0; c < 4; ++c) {
                            const int f1 = 16 * j + 8 * pr + 4 * g + c;
                            Tr<EL>::store(slab, kcache_index<EL, D>(pos, f1), lo_v[pr][c]);
                            Tr<EL>::store(slab, kcache_index<EL, D>(pos, f1 + D / 2), hi_v[pr][c]);
                        }
                }
            } else if (t < a.T) {
                const int kh = head - a.Hq - a.Hkv;
                char* slab = (char*)a.vcache + (size_t)kh * a.S_pad * D * Tr<EL>::ESZ;
                const int pos = a.L + t;
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int f = 32 * j + 8 * (i >> 2) + 4 * g + (i & 3);
                    Tr<EL>::store(slab, vcache_index<EL, D>(pos, f), acc[i]);
                }
            }
        }
    }
}

// ============================================================================ tree attention
// For node t and query head qh: softmax over {cache slots 0..L-1} U {tree slots L+j : j in
// ancestors-or-self(t)} of q.k/sqrt(D), times V.  A workgroup handles one (query head,
// block of 32 nodes); its four wavefronts take every fourth 32-key block, keep online-softmax
// statistics, and are merged through LDS.  Scores are computed transposed (keys x nodes)
// so that each lane owns one node: the node's 256-bit ancestor set sits in registers and
// is tested per key, and the probabilities are already in B-operand order for V^T * P^T.
struct AttnArgs {
    const uint4* q;          // vector-major [Hq*D/E][Tp]
    const uint4* kc;         // this layer's K slabs
    const uint4* vc;
    void* out;               // vector-major [Hq*D/E][Tp]
    const uint64_t* mask;    // [Tp][4]
    int Tp, T, L, Hq, Hkv, S_pad;
    float scale;
};

template <typename EL, int D>
__global__ __launch_bounds__(256) void k_attn(AttnArgs a) {
    constexpr int E = Tr<EL>::E;
    constexpr int NF = D / (2 * E);      // K frags per key block
    constexpr int NQ = 32 / (2 * E);     // V frags per (key block, 32 features)
    constexpr int DB = D / 32;
    __shared__ float smem[3 * DB * 64 * 16 + 8 * 32];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int tl = lane & 31, g = lane >> 5;
    const int TB = a.Tp >> 5;
    const int qh = blockIdx.x / TB, tb = blockIdx.x % TB;
    const int kh = qh / (a.Hq / a.Hkv);
    const int t = tb * 32 + tl;

    uint4 qf[NF];
#pragma unroll
    for (int fr = 0; fr < NF; ++fr) qf[fr] = a.q[((size_t)(qh * (D / E) + 2 * fr + g)) * a.Tp + t];
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

    const int n_keys = a.L + a.T;
    const int nkb = (n_keys + 31) >> 5;
    const int lidx = tl * 2 + g;   // position of this lane's 16 bytes inside a 1 KiB tile
    for (int kb = wave; kb < nkb; kb += 4) {
        floatx16 s;
#pragma unroll
        for (int i = 0; i < 16; ++i) s[i] = 0.f;
        const uint4* kp = kslab + (size_t)kb * NF * 64 + lidx;
#pragma unroll
        for (int fr = 0; fr < NF; ++fr) s = Tr<EL>::mma(kp[fr * 64], qf[fr], s);

        float p[16];
        float mx = -1e30f;
        const bool all_prefix = (kb * 32 + 32 <= a.L);
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int key = kb * 32 + 8 * (i >> 2) + 4 * g + (i & 3);
            bool vis = true;
            if (!all_prefix) {
                const int n = key - a.L;   // tree index of this key if >= 0
                vis = (n < 0) || (n < a.T && ((mk[(n >> 6) & 3] >> (n & 63)) & 1ull));
            }
            p[i] = vis ? s[i] * a.scale : -1e30f;
            mx = fmaxf(mx, p[i]);
        }
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(m_run, mx);
        const float alpha = __expf(m_run - m_new);
        float psum = 0.f;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            p[i] = (p[i] > -1e29f) ? __expf(p[i] - m_new) : 0.f;
            psum += p[i];
        }
        l_run = l_run * alpha + psum;
        m_run = m_new;
        uint4 pb[NQ];
#pragma unroll
        for (int q = 0; q < NQ; ++q) pb[q] = Tr<EL>::pack(p + q * E);
        const uint4* vp = vslab + (size_t)kb * DB * NQ * 64 + lidx;
#pragma unroll
        for (int db = 0; db < DB; ++db) {
#pragma unroll
            for (int i = 0; i < 16; ++i) o[db][i] *= alpha;
#pragma unroll
            for (int q = 0; q < NQ; ++q) o[db] = Tr<EL>::mma(vp[(db * NQ + q) * 64], pb[q], o[db]);
        }
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
    if (wave != 0) return;
    float M = -1e30f;
#pragma unroll
    for (int w = 0; w < 4; ++w) M = fmaxf(M, sm[w * 32 + tl]);
    float wgt[4], lsum = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) { wgt[w] = __expf(sm[w * 32 + tl] - M); lsum += wgt[w] * sl[w * 32 + tl]; }
    const float inv = (lsum > 0.f) ? 1.f / lsum : 0.f;
#pragma unroll
    for (int db = 0; db < DB; ++db) {
        float r[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) r[i] = wgt[0] * o[db][i];
#pragma unroll
        for (int w = 1; w < 4; ++w)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float4 v = ((const float4*)so)[(((w - 1) * DB + db) * 64 + lane) * 4 + q];
                r[4 * q] += wgt[w] * v.x; r[4 * q + 1] += wgt[w] * v.y; r[4 * q + 2] += wgt[w] * v.z; r[4 * q + 3] += wgt[w] * v.w;
            }
#pragma unroll
        for (int blk = 0; blk < 4; ++blk)
            store4_act<EL>(a.out, a.Tp, qh * D + db * 32 + 8 * blk + 4 * g, t, r[4 * blk] * inv, r[4 * blk + 1] * inv,
                           r[4 * blk + 2] * inv, r[4 * blk + 3] * inv);
    }
}

// ============================================================================ argmax
// Greedy choice per node: wavefront shuffle reduction on (value, index), lowest index on ties.
struct ArgmaxArgs {
    const float* logits;   // [Tp][Vpad]
    int32_t* am;           // [Tp]
    int V, Vpad;
};

__device__ __forceinline__ void argmax_combine(float& v, int& i, float ov, int oi) {
    if (ov > v || (ov == v && oi < i)) { v = ov; i = oi; }
}

__global__ __launch_bounds__(256) void k_argmax(ArgmaxArgs a) {
    __shared__ float sv[4];
    __shared__ int si[4];
    const int t = blockIdx.x, tid = threadIdx.x;
    const float* row = a.logits + (size_t)t * a.Vpad;
    float bv = -INFINITY;
    int bi = 0x7fffffff;
    for (int v0 = tid * 4; v0 < a.V; v0 += 256 * 4) {
        const float4 x = *(const float4*)(row + v0);
        const float xs[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
        for (int c = 0; c < 4; ++c)
            if (v0 + c < a.V) argmax_combine(bv, bi, xs[c], v0 + c);
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const float ov = __shfl_xor(bv, off);
        const int oi = __shfl_xor(bi, off);
        argmax_combine(bv, bi, ov, oi);
    }
    if ((tid & 63) == 0) { sv[tid >> 6] = bv; si[tid >> 6] = bi; }
    __syncthreads();
    if (tid == 0) {
        for (int w = 1; w < 4; ++w) argmax_combine(bv, bi, sv[w], si[w]);
        a.am[t] = bi;
    }
}

// ============================================================================ longest accepted path
// Single block.  match[i] = (i is the root) or tok[i] == argmax[parent[i]]; node i is
// accepted iff every node of its ancestor set matches; best = deepest accepted node, lowest
// index among equals; path = members of best's ancestor set in increasing index (= depth) order.
struct FvResult {
    int32_t accepted_len, next_token, best, pad;
    int32_t path[FV_MAX_TREE];
    int32_t accepted_tokens[FV_MAX_TREE];
};

struct ScanArgs {
    const int32_t* tok_in;   // [3][cap]
    int cap, T;
    const uint64_t* mask;
    const int32_t* am;
    FvResult* res;
};

__global__ __launch_bounds__(256) void k_scan(ScanArgs a) {
    __shared__ unsigned long long mbits[4];
    __shared__ int best_key;
    const int i = threadIdx.x;
    const int32_t* tok = a.tok_in;
    const int32_t* parent = a.tok_in + a.cap;
    const int32_t* depth = a.tok_in + 2 * a.cap;
    if (i < 4) mbits[i] = 0ull;
    if (i == 0) best_key = -1;
    __syncthreads();
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
enum { TILE_NAT = 0, TILE_QKV = 1, TILE_GU = 2 };
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
    const size_t fb = idx >> 6;
    const int frag = (int)(fb % ((size_t)a.NB * FV_FRAGS));
    const int strip = (int)(fb / ((size_t)a.NB * FV_FRAGS));
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
