// Tree attention in a form whose result for a node does not depend on the step it is computed in.
//
// The paper's claim is that drafting plus verification emits exactly what plain decoding emits
// (Abstract; section "Custom-Designed Decoding Tree").  In floating point that needs more than the
// right mask: a node must get bitwise the same attention output when it is verified alone (one
// token per step) and as one of 64 tree nodes, or a top-2 near-tie can tip the two ways.  k_attn
// does not give that: how the keys are divided among wavefronts and workgroups depends on the
// step's row count, and a node's ancestors sit at cache slots L + ancestor index inside a tree step
// but at consecutive slots in plain decoding, so they meet the fp32 sums in different positions.
//
// Here every operation on node t is a function of its sequence position p = L + depth alone:
//
//  * FAR keys, positions [0, 32 * nfb), nfb = max(0, p / 32 - 1).  Always cache slots below L (they
//    are committed tokens in either kind of step: a node is at most FV_CANON_DEPTH = 32 deep).  They
//    are cut into PARTS at fixed absolute positions: parts 0-3 hold 4 blocks of 32 keys, parts 4-7
//    8 blocks, parts 8-11 16, later ones 32.  The four wavefronts of a workgroup take a quarter of a
//    part each (a run of 1, 2, 4 or 8 consecutive blocks, online softmax inside the run, the
//    rescale decision per node), are merged through LDS in wavefront order, and the part's (max, sum,
//    output) triple goes to the part's own slot.  Which workgroup computes which part is scheduling
//    only.  A block at or beyond a node's own nfb is invisible to it as a whole and contributes
//    exact zeros, so a step that holds deeper nodes (more parts) changes nothing for this one.
//  * WINDOW keys, positions [32 * nfb, p]: at most 64, one per lane, in position order whatever
//    slots they occupy (prefix slots, then the node's ancestors by depth).  Their scores come from
//    shared matrix tiles (a score does not depend on its key's slot); the softmax denominator and
//    the weighted sum of V rows are fp32 vector arithmetic per node in a fixed order (see
//    canon_window); the result is one more triple in the slot after the last part.
//  * The last workgroup of an item to arrive merges the slots in slot order.
//
// The matrix cores see the far keys exactly as in k_attn (K and V tiles straight from the cache
// layout, q and the probabilities as hi + lo bf16 pairs).
#pragma once
// (included from fv_kernels.hpp after attn_body)

struct CanonArgs {
    const uint4* q;          // vector-major [Hq*D/E][Tp]
    const uint4* q_lo;       // bf16 only
    const uint4* kc;         // this layer's K slabs
    const uint4* vc;
    void* out;               // vector-major [Hq*D/E][Tp]
    const int32_t* pos;      // [Tp] sequence position L + depth of every row
    const uint8_t* anc;      // [Tp][FV_CANON_DEPTH + 1]: row t's ancestor at depth d (itself at its own depth)
    int Tp, T, L, Hq, Hkv, S_pad;
    float scale;
    int nfb;                 // far blocks of the deepest row of the step (32 * nfb <= L)
    int np;                  // far parts: canon_parts(nfb)
    int kw;                  // workgroups per (head, node block) item
    unsigned char owner[FV_CANON_MAX_PARTS];   // part -> workgroup of the item that computes it
    float* part;             // [item][np + 1][FV_ATTN_PART_FLOATS]
    int* tickets;            // [item], zero on entry, left zero
};

// LDS of the window: the scores of every (node, window slot) pair as fp32 [32 nodes][FV_CANON_SROW]
// (an odd row length: the lanes of a score tile write one node each), and the V tiles of the
// window's key blocks in the cache's own order, every 16-byte vector at a stride of 24 bytes so
// that lanes reading one position of 64 different features hit different banks.  The far parts'
// merge area reuses the same bytes afterwards.
#define FV_CANON_WIN_BLOCKS 4    // key blocks the windows of one step can touch: L/32 - 1 .. (L + 63)/32
#define FV_CANON_SROW (FV_CANON_WIN_BLOCKS * 32 + 1)
#define FV_CANON_VSTRIDE 24
#define FV_CANON_WIN_BYTES(D, ESZ) \
    (32 * FV_CANON_SROW * 4 + FV_CANON_WIN_BLOCKS * ((D) / 32) * (ESZ) * 64 * FV_CANON_VSTRIDE)   /* NQ = 32 / (2E) = ESZ */
#define FV_CANON_SMEM_BYTES(D, ESZ) \
    (FV_CANON_WIN_BYTES(D, ESZ) > FV_ATTN_SMEM_FLOATS(D) * 4 ? FV_CANON_WIN_BYTES(D, ESZ) : FV_ATTN_SMEM_FLOATS(D) * 4)

// Wavefront-wide maximum and sum through the cross-lane data path (no LDS round trips): four steps
// inside each row of 16 lanes, then row 0 into 1 and 2 into 3, then the lower half into the upper;
// lane 63 holds the result.  One fixed tree: the sum of a window is the same bits in every step.
template <int CTRL, int ROWS>
__device__ __forceinline__ float canon_dpp(float identity, float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(__builtin_bit_cast(int, identity), __builtin_bit_cast(int, v),
                                                                 CTRL, ROWS, 0xf, false));
}
__device__ __forceinline__ float canon_wave_max(float v) {
    v = fmaxf(v, canon_dpp<0xB1, 0xf>(-1e30f, v));    // quad_perm [1,0,3,2]
    v = fmaxf(v, canon_dpp<0x4E, 0xf>(-1e30f, v));    // quad_perm [2,3,0,1]
    v = fmaxf(v, canon_dpp<0x141, 0xf>(-1e30f, v));   // row_half_mirror
    v = fmaxf(v, canon_dpp<0x140, 0xf>(-1e30f, v));   // row_mirror
    v = fmaxf(v, canon_dpp<0x142, 0xa>(-1e30f, v));   // row_bcast 15 into rows 1 and 3
    v = fmaxf(v, canon_dpp<0x143, 0xc>(-1e30f, v));   // row_bcast 31 into rows 2 and 3
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}
__device__ __forceinline__ float canon_wave_sum(float v) {
    v += canon_dpp<0xB1, 0xf>(0.f, v);
    v += canon_dpp<0x4E, 0xf>(0.f, v);
    v += canon_dpp<0x141, 0xf>(0.f, v);
    v += canon_dpp<0x140, 0xf>(0.f, v);
    v += canon_dpp<0x142, 0xa>(0.f, v);
    v += canon_dpp<0x143, 0xc>(0.f, v);
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}

// What a window job reads from global memory: requested one job ahead, so that its round trip is
// hidden behind the score tiles (first job) or the previous job's arithmetic.
struct CanonJob { int p; int anc; };
__device__ __forceinline__ CanonJob canon_job_load(const CanonArgs& a, int t, int lane) {
    CanonJob jb;
    jb.p = 0; jb.anc = 0;
    if (t < a.T) {
        jb.p = a.pos[t];
        jb.anc = (lane <= FV_CANON_DEPTH) ? a.anc[t * (FV_CANON_DEPTH + 1) + lane] : 0;   // lane d: the ancestor at depth d
    }
    return jb;
}

// The window triples of nodes [n0, n1) of the item, one wavefront per node.
//
// Scores do not care where a key sits: score(key, node) is one dot product over the features, the same bits in
// whatever tile row the key's slot puts it.  So the scores of all 32 nodes against every slot of the window's key
// blocks come from shared matrix tiles exactly as for the far keys (qf, qfl: this lane's q operand, hi and lo), and go
// to LDS.  What has to follow the positions is the order of the sums: the softmax denominator and the weighted sum of V
// rows, done per node by one wavefront -- lane j takes the node's j-th window position (looking its slot up: prefix
// slots, then ancestors by depth), the denominator is one fixed tree over the lanes, and the output adds the positions
// in ascending order, each lane for D/64 features, reading V straight from the staged tiles.
template <typename EL, int D, int NFQ>
__device__ __forceinline__ void canon_window(const CanonArgs& a, const uint4 (&qf)[NFQ], const uint4 (&qfl)[NFQ], int kh, int tb,
                                             int n0, int n1, char* lds, float* slot) {
    constexpr int E = Tr<EL>::E, ESZ = Tr<EL>::ESZ;
    constexpr int NF = D / (2 * E), NQ = 32 / (2 * E), DB = D / 32;
    constexpr int FPL = D / 64;            // output features per lane: lane, lane + 64
    constexpr bool SPLIT = (E == 8);
    constexpr int VPB = DB * NQ * 64;      // V vectors per key block
    constexpr int VIT = (FV_CANON_WIN_BLOCKS * VPB + 255) / 256;
    constexpr int VST = FV_CANON_VSTRIDE;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int tl = lane & 31, g = lane >> 5;
    float* Sl = (float*)lds;
    char* Vl = lds + 32 * FV_CANON_SROW * 4;
    const int lb = a.L >> 5;
    const int pb0 = lb > 0 ? lb - 1 : 0, pb1 = (a.L + a.T - 1) >> 5;   // key blocks the windows touch (at most four)
    const int WS0 = 32 * pb0;
    const size_t slab_vecs = (size_t)a.S_pad * D / E;
    const uint4* kslab = a.kc + (size_t)kh * slab_vecs;
    const uint4* vslab = a.vc + (size_t)kh * slab_vecs;

    // ---- requests: the K tiles of this wavefront's window block, the V tiles of all window blocks, the first job's data
    const int kbw = pb0 + wave;
    uint4 kt[NF];
    if (kbw <= pb1) {
        const uint4* kp = kslab + (size_t)kbw * NF * 64 + tl * 2 + g;
#pragma unroll
        for (int fr = 0; fr < NF; ++fr) kt[fr] = kp[fr * 64];
    }
    const int nvv = (pb1 - pb0 + 1) * VPB;
    uint4 vst[VIT];
#pragma unroll
    for (int it = 0; it < VIT; ++it) {
        const int idx = tid + it * 256;
        if (idx < nvv) vst[it] = vslab[(size_t)pb0 * VPB + idx];
    }
    CanonJob cur = canon_job_load(a, tb * 32 + n0 + wave, lane);

    // ---- score tile of this wavefront's block: keys x nodes, to LDS as [node][slot - WS0]
    if (kbw <= pb1) {
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
        float* sp = Sl + tl * FV_CANON_SROW + (kbw - pb0) * 32 + 4 * g;
#pragma unroll
        for (int i = 0; i < 16; ++i) sp[8 * (i >> 2) + (i & 3)] = (s[i] + s1[i]) * a.scale;
    }
#pragma unroll
    for (int it = 0; it < VIT; ++it) {
        const int idx = tid + it * 256;
        if (idx < nvv) {
            uint64_t* d = (uint64_t*)(Vl + (size_t)idx * VST);
            d[0] = (uint64_t)vst[it].x | ((uint64_t)vst[it].y << 32);
            d[1] = (uint64_t)vst[it].z | ((uint64_t)vst[it].w << 32);
        }
    }
    __syncthreads();

    for (int n = n0 + wave; n < n1; n += 4) {
        const int t = tb * 32 + n;
        const CanonJob jb = cur;
        if (n + 4 < n1) cur = canon_job_load(a, t + 4, lane);
        float m = -1e30f, l = 0.f, acc[FPL];
#pragma unroll
        for (int i = 0; i < FPL; ++i) acc[i] = 0.f;
        if (t < a.T) {   // wavefront-uniform
            const int p = jb.p;
            const int pbk = p >> 5;
            const int ws = 32 * (pbk > 0 ? pbk - 1 : 0);
            const int nw = p - ws + 1;                 // window positions, 1 .. 64
            const bool valid = lane < nw;
            const int pj0 = ws + lane;
            const int anc_j = __shfl(jb.anc, (pj0 - a.L) & 63);   // tree positions: the ancestor at depth pj - L
            const int sj = valid ? (pj0 < a.L ? pj0 : a.L + anc_j) : WS0;   // this lane's slot
            const float sc = valid ? Sl[n * FV_CANON_SROW + (sj - WS0)] : -1e30f;
            m = canon_wave_max(sc);
            const float pj = valid ? __expf(sc - m) : 0.f;   // zero beyond the window: those lanes add nothing below
            l = canon_wave_sum(pj);
            // byte offset of this lane's position inside the staged V tiles, for feature 0 of the block of 32 features:
            // vector ((db * NQ + q) * 32 + f) * 2 + g of the key block, element e
            const int pp = sj & 31, ii = 4 * (pp >> 3) + (pp & 3);
            const int voff = ((((sj >> 5) - pb0) * VPB + (ii / E) * 64 + ((pp >> 2) & 1)) * VST) + (ii % E) * ESZ;
            const char* vl = Vl + (((lane >> 5) * NQ * 64) + (lane & 31) * 2) * VST;   // feature `lane`: block lane / 32, row lane % 32
            // output: positions in ascending order, eight of them requested at a time
            for (int j0 = 0; j0 < nw; j0 += 8) {
                float w[8], vf[8][FPL];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int j = (j0 + u) & 63;
                    w[u] = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, pj), j));
                    const char* vr = vl + __builtin_amdgcn_readlane(voff, j);
#pragma unroll
                    for (int i = 0; i < FPL; ++i) {   // feature lane + 64 i: two blocks of 32 features further on
                        const char* ve = vr + i * (2 * NQ * 64 * VST);
                        if constexpr (E == 8) vf[u][i] = bf16_bits_to_f32(*(const uint16_t*)ve); else vf[u][i] = *(const float*)ve;
                    }
                }
#pragma unroll
                for (int u = 0; u < 8; ++u)
#pragma unroll
                    for (int i = 0; i < FPL; ++i) acc[i] = fmaf(w[u], vf[u][i], acc[i]);
            }
        }
        // the triple, in the layout of the far parts' triples (accumulator order of the 32x32 tiles)
#pragma unroll
        for (int i = 0; i < FPL; ++i) {
            const int f = lane + 64 * i, fm = f & 31;
            const int reg = 4 * (fm >> 3) + (fm & 3), gg = (fm >> 2) & 1;
            __hip_atomic_store(slot + ((f >> 5) * 16 + reg) * 64 + gg * 32 + n, acc[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        if (lane == 0) {
            __hip_atomic_store(slot + DB * 1024 + n, m, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(slot + DB * 1024 + 32 + n, l, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

// Workgroup k of the kw that share item (query head, block of 32 nodes).
template <typename EL, int D>
__device__ __forceinline__ void attn_canon_body(const CanonArgs& a, int item, int k, char* lds) {
    constexpr int E = Tr<EL>::E;
    constexpr int NF = D / (2 * E), NQ = 32 / (2 * E), DB = D / 32;
    constexpr int PF = FV_ATTN_PART_FLOATS(D);
    constexpr bool SPLIT = (E == 8);
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int tl = lane & 31, g = lane >> 5;
    const int TB = a.Tp >> 5;
    const int qh = item / TB, tb = item % TB;
    const int kh = qh / (a.Hq / a.Hkv);
    const int t = tb * 32 + tl;
    float* slots = a.part + (size_t)item * (a.np + 1) * PF;

    // Everything the far parts read from global memory before their first matrix product is requested
    // now, ahead of the window, so that the kernel pays that round trip once: q, and the K and V tiles
    // of the first block of this wavefront's first run.
    int j_first = -1;
    for (int j = a.np - 1; j >= 0; --j) if (a.owner[j] == k) j_first = j;
    const bool mine = j_first >= 0;
    uint4 qf[NF], qfl[NF];   // (qfl is not used by fp32 builds)
    uint4 kt0[NF], vt0[DB * NQ];
    const size_t slab_vecs = (size_t)a.S_pad * D / E;
    const uint4* kslab = a.kc + (size_t)kh * slab_vecs;
    const uint4* vslab = a.vc + (size_t)kh * slab_vecs;
    const int lidx = tl * 2 + g;
    auto load_block = [&](uint4 (&kt)[NF], uint4 (&vt)[DB * NQ], int kb) {
        const uint4* kp = kslab + (size_t)kb * NF * 64 + lidx;
        const uint4* vp = vslab + (size_t)kb * DB * NQ * 64 + lidx;
#pragma unroll
        for (int fr = 0; fr < NF; ++fr) kt[fr] = kp[fr * 64];
#pragma unroll
        for (int jj = 0; jj < DB * NQ; ++jj) vt[jj] = vp[jj * 64];
    };
    int p_t = 0;
    int pre_kb = -1;   // the key block whose tiles kt0, vt0 hold
#pragma unroll
    for (int fr = 0; fr < NF; ++fr) qf[fr] = a.q[((size_t)(qh * (D / E) + 2 * fr + g)) * a.Tp + t];
    if constexpr (SPLIT) {
#pragma unroll
        for (int fr = 0; fr < NF; ++fr) qfl[fr] = a.q_lo[((size_t)(qh * (D / E) + 2 * fr + g)) * a.Tp + t];
    }
    if (mine) {
        p_t = (t < a.T) ? a.pos[t] : 0;
        const int kb = canon_part_b0(j_first) + wave * canon_part_run(j_first);
        if (kb < a.nfb) { load_block(kt0, vt0, kb); pre_kb = kb; }
    }

    canon_window<EL, D, NF>(a, qf, qfl, kh, tb, 32 * k / a.kw, 32 * (k + 1) / a.kw, lds, slots + (size_t)a.np * PF);
    __syncthreads();   // the far parts reuse the window's LDS

    float* smem = (float*)lds;
    float* so = smem;                              // [3][DB][64][16]
    float* sm = smem + 3 * DB * 64 * 16;           // [4][32] reference maxima
    float* sl = sm + 4 * 32;                       // [4][32] sums
    int* ticket_lds = (int*)(sl + 4 * 32);

    if (mine) {
        const int nfb_t = (t < a.T && (p_t >> 5) > 0) ? (p_t >> 5) - 1 : 0;   // this node's far blocks
        for (int j = j_first; j < a.np; ++j) {
            if (a.owner[j] != k) continue;
            const int run = canon_part_run(j), kb0 = canon_part_b0(j) + wave * run;
            floatx16 o[DB];
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int i = 0; i < 16; ++i) o[db][i] = 0.f;
            float m_run = -1e30f, l_run = 0.f;
            for (int kb = kb0; kb < kb0 + run && kb < a.nfb; ++kb) {
                uint4 kt[NF], vt[DB * NQ];
                if (pre_kb == kb) {   // requested ahead of the window
#pragma unroll
                    for (int fr = 0; fr < NF; ++fr) kt[fr] = kt0[fr];
#pragma unroll
                    for (int jj = 0; jj < DB * NQ; ++jj) vt[jj] = vt0[jj];
                } else {
                    load_block(kt, vt, kb);
                }
                __builtin_amdgcn_sched_barrier(0);
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
                const bool vis = kb < nfb_t;   // a far block is visible to a node as a whole or not at all
                float p[16];
                float mx = -1e30f;
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    p[i] = vis ? s[i] * a.scale : -1e30f;
                    mx = fmaxf(mx, p[i]);
                }
                mx = fmaxf(mx, __shfl_xor(mx, 32));
                // the reference only has to stay within 8 of the running maximum; whether it moves is decided per
                // node (a lane that stays put multiplies by exactly one), so a node's sums do not depend on its neighbours
                const float m_cand = fmaxf(m_run, mx);
                const bool trig = m_cand - m_run > 8.f;
                if (__any(trig)) {
                    const float alpha = trig ? __expf(m_run - m_cand) : 1.f;
                    l_run *= alpha;
                    if (trig) m_run = m_cand;
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
                if constexpr (SPLIT) {
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
            }
            l_run += __shfl_xor(l_run, 32);

            // the four quarters of the part, in wavefront order
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
            if (wave == 0) {
                float M = -1e30f, lsum = 0.f;
#pragma unroll
                for (int w = 0; w < 4; ++w) M = fmaxf(M, sm[w * 32 + tl]);
                float wgt[4];
#pragma unroll
                for (int w = 0; w < 4; ++w) { wgt[w] = __expf(sm[w * 32 + tl] - M); lsum += wgt[w] * sl[w * 32 + tl]; }
                float* pp = slots + (size_t)j * PF + lane;
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
                            r[4 * q] += wgt[w] * v.x; r[4 * q + 1] += wgt[w] * v.y;
                            r[4 * q + 2] += wgt[w] * v.z; r[4 * q + 3] += wgt[w] * v.w;
                        }
#pragma unroll
                    for (int i = 0; i < 16; ++i) __hip_atomic_store(pp + (db * 16 + i) * 64, r[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
                if (g == 0) {
                    __hip_atomic_store(pp + DB * 1024, M, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);         // lanes 0..31
                    __hip_atomic_store(pp + DB * 1024 + 32, lsum, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            }
            __syncthreads();   // the merge area is reused by the next part
        }
    }

    // ---- every triple of this workgroup is acknowledged, then the ticket; the last arriver merges the slots
    handoff_release();
    __syncthreads();
    if (tid == 0) *ticket_lds = __hip_atomic_fetch_add(&a.tickets[item], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    handoff_acquire();
    if (*ticket_lds != a.kw - 1) return;
    if (tid == 0) __hip_atomic_store(&a.tickets[item], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // for the next use
    const int ns = a.np + 1;
    for (int db = wave; db < DB; db += 4) {
        // slot order; the common reference is the largest of the slots' references.  Up to eight slots are requested
        // in one go (the merge then costs one memory round trip); beyond that the references are read first.
        float Mx = -1e30f;
        if (ns > 8)
            for (int c = 0; c < ns; ++c)
                Mx = fmaxf(Mx, __hip_atomic_load(slots + (size_t)c * PF + DB * 1024 + tl, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
        float accv[16], ltot = 0.f;
#pragma unroll
        for (int i = 0; i < 16; ++i) accv[i] = 0.f;
        for (int c0 = 0; c0 < ns; c0 += 8) {
            float mc[8], lc[8], v[8][16];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const float* cp = slots + (size_t)(c0 + u < ns ? c0 + u : 0) * PF;
                mc[u] = __hip_atomic_load(cp + DB * 1024 + tl, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                lc[u] = __hip_atomic_load(cp + DB * 1024 + 32 + tl, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
                for (int i = 0; i < 16; ++i) v[u][i] = __hip_atomic_load(cp + (db * 16 + i) * 64 + lane, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            if (ns <= 8) {
#pragma unroll
                for (int u = 0; u < 8; ++u) if (u < ns) Mx = fmaxf(Mx, mc[u]);
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                if (c0 + u < ns) {   // wavefront-uniform
                    const float wc = __expf(mc[u] - Mx);
                    ltot += wc * lc[u];
#pragma unroll
                    for (int i = 0; i < 16; ++i) accv[i] += wc * v[u][i];
                }
            }
        }
        const float inv = (ltot > 0.f) ? 1.f / ltot : 0.f;
#pragma unroll
        for (int blk = 0; blk < 4; ++blk)
            store4_act<EL>(a.out, a.Tp, qh * D + db * 32 + 8 * blk + 4 * g, t, accv[4 * blk] * inv, accv[4 * blk + 1] * inv,
                                accv[4 * blk + 2] * inv, accv[4 * blk + 3] * inv);
    }
}

// grid = items * kw, dynamic LDS FV_CANON_SMEM_BYTES
template <typename EL, int D>
__global__ __launch_bounds__(256) void k_attn_canon(CanonArgs a) {
    extern __shared__ __attribute__((aligned(16))) char lds_dyn[];
    // all workgroups of a query head (and of the heads that share its KV head) on one XCD, as in k_attn
    int item = blockIdx.x / a.kw, k = blockIdx.x % a.kw;
    if ((a.Hq & 7) == 0) {
        const int x = blockIdx.x & 7, j = blockIdx.x >> 3;
        const int TB = a.Tp >> 5, per_head = TB * a.kw;
        const int head = x * (a.Hq >> 3) + j / per_head, w = j % per_head;
        item = head * TB + w / a.kw;
        k = w % a.kw;
    }
    attn_canon_body<EL, D>(a, item, k, lds_dyn);
}
