// Skinny GEMM for up to 64 tokens, "direct" form: one 32-row strip (RS = 1) or a pair of strips
// (RS = 2, a 64-row group) per workgroup at a time, three wavefronts split the K range of that
// row group between them, and both MFMA operands go straight from global memory to registers
// (weights from HBM, activations from L2): no LDS and no workgroup barrier inside the streaming
// loop, so every streaming wavefront runs its own software pipeline.  The fourth wavefront streams
// nothing; it adds up the others' sums where a segment ends.
//
// Work split: the (row group, K stage) space is cut into G contiguous ranges, one per workgroup
// (equal stream-K ranges, or whole row groups when the host says `aligned`).  The part of a range
// inside one row group is a segment; a streaming wavefront's third of a segment is a slice.  At the
// end of a segment the streaming wavefronts put their accumulators into LDS, where they are added
// in wavefront order and the sum is parked.  Nothing leaves the compute unit before the range ends.
// Then a segment that covers the whole K range goes to the epilogue; of a row group shared by
// several workgroups, every contributor but the first stores its partial tiles with a mark in the
// lowest mantissa bit of every value, and the first contributor waits (a bounded number of looks)
// until all of them are marked, adds them in ascending workgroup order, writes zeros back and runs
// the epilogue.  The partial area is all zeros when a launch starts and when it ends.
//
// A stage is 8 weight tiles of 1 KiB: RS = 1: 8 fragments of one strip (a K batch) with 8*TB
// activation tiles; RS = 2: 4 fragments of each of two strips (half a K batch) with 4*TB
// activation tiles.  Tiles are requested three stages ahead into three rotating register sets in a
// fixed issue order, so the hardware's in-order load counter lets each wait be exact.
//
// The streaming loop is kept to the instructions that matter.  With one wavefront per SIMD nothing
// hides instruction issue, and an earlier form of this loop (a general cursor advanced three times
// per stage, accumulators shuttled between the two register files around a conditional) spent
// more cycles on bookkeeping than on waiting for HBM.  Now: every slice is padded to whole rounds
// of three stages; a padded stage loads 16 bytes of zeros per instruction instead of tiles, so
// its MFMAs add nothing and the loop body has no conditional at all; addresses advance by
// constants inside a slice and are recomputed only when the request stream enters the next slice.
#pragma once
// (included from fv_kernels.hpp after GemmArgs, gemm_epilogue and zero_acc)


// Shared-memory needs, in floats: two accumulator exchange areas [3 streaming wavefronts][tiles][16][64]
// (used alternately from segment to segment), RMSNorm factors [Tp], reduction scratch [1024], 4 spare words,
// parked sums [FV_PARK][tiles][16][64].
#define FV_STREAMERS 3   // wavefronts 0..2 stream; wavefront 3 adds up their sums at the ends of segments
#define FV_PARK 3        // reduced tiles of this many segments are kept in LDS before anything is stored
#define FV_DIRECT_SMEM_FLOATS(TB) ((2 * FV_STREAMERS + FV_PARK) * (TB) * 1024 + (TB) * 32 + 1024 + 4)
#define FV_PAIRED_SMEM_FLOATS(TB) ((2 * FV_STREAMERS + FV_PARK) * 2 * (TB) * 1024 + (TB) * 32 + 1024 + 4)

// This workgroup's range of the (row group, K stage) space and this wavefront's slices of it.
struct DPlan {
    int u0, u1, g0, nseg, NB, wave;
    __device__ __forceinline__ void init(const GemmArgs& a, int wg, int wave_) {
        // computed, not looked up: a table read would put one more memory round trip in front of
        // the first weight load
        // (32-bit arithmetic: the host only selects these kernels when NG * NB * G < 2^31; G is a
        // power of two whenever there is at least one unit per compute unit, and then a shift)
        const unsigned G = (unsigned)a.G;
        const bool pow2 = (G & (G - 1)) == 0;
        const int sh = 31 - __builtin_clz(G);
        auto divG = [&](unsigned v) { return pow2 ? (v >> sh) : v / G; };
        if (a.aligned) {   // whole row groups per workgroup: counts differ by at most one
            u0 = (int)divG((unsigned)(a.NG * wg)) * a.NB;
            u1 = (int)divG((unsigned)(a.NG * (wg + 1))) * a.NB;
        } else {
            const unsigned U = (unsigned)(a.NG * a.NB);
            u0 = (int)divG(U * (unsigned)wg);
            u1 = (int)divG(U * (unsigned)(wg + 1));
        }
        NB = a.NB; wave = wave_;
        g0 = u0 / NB;
        nseg = 1;
        for (int e_ = (g0 + 1) * NB; e_ < u1; e_ += NB) ++nseg;
    }
    // segment s: row group gi, stages [b0, b0 + nb)
    __device__ __forceinline__ void segment(int s, int& gi, int& b0, int& nb) const {
        gi = g0 + s;
        b0 = (s == 0) ? u0 - g0 * NB : 0;
        const int rem = u1 - gi * NB;
        nb = (rem < NB ? rem : NB) - b0;
    }
    // this wavefront's third [ws, we) of segment s
    __device__ __forceinline__ void slice(int s, int& gi, int& ws, int& we) const {
        int b0, nb;
        segment(s, gi, b0, nb);
        if (wave >= FV_STREAMERS) { ws = we = b0 + nb; return; }   // the fourth wavefront streams nothing
        ws = b0 + nb * wave / FV_STREAMERS;
        we = b0 + nb * (wave + 1) / FV_STREAMERS;
    }
};

// Request stream of one wavefront: the stages of its slices in order, every slice padded to a
// multiple of three stages.  (wp, xp) are this lane's addresses for the current stage; past the
// real stages of a slice, and past the last slice, `live` is false and the loads read zeros.
struct DReq {
    int s;          // slice (= segment) being requested; nseg when the stream has ended
    int j, n, n3;   // padded stage index inside the slice, real stages, padded stages
    const uint4* wp;
    const uint4* xp;
};

// `wg` is this workgroup's index in the split.
template <typename EL, int TB, int D, int EPI, int RS = 1>
__device__ __forceinline__ void gemm_direct_body(const GemmArgs& a, int wg, float* smem) {
    constexpr int Tp = TB * 32;
    constexpr int SF = FV_FRAGS / RS;            // fragments per stage
    constexpr int NX = SF * TB;                  // activation tiles per stage
    constexpr int NT = RS * TB;                  // accumulator tiles per wavefront
    static_assert(RS == 1 || RS == 2, "one or two strips per wavefront");
    float* red = smem;                           // [2][streaming wavefront][tile][16][64]
    float* rinv_lds = red + 2 * FV_STREAMERS * NT * 1024;
    float* red_lds = rinv_lds + Tp;              // 16-byte aligned: Tp is a multiple of 32
    constexpr bool with_norm = EPI != EPI_RESID;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int tl = lane & 31, g = lane >> 5;
    if (wg >= a.G) return;
    FV_TS(0)

    // RMSNorm factor of every token from the [n_ssq][Tp] partial sums of squares.  These loads go out
    // before anything else (L2 hits; the work-split arithmetic below runs while they are in flight),
    // the weight/activation prefetch right behind them, the cross-thread reduction after that.
    float4 s4 = make_float4(0.f, 0.f, 0.f, 0.f);
    float4 sv[8];   // the first (usually only) eight rows of this thread: summed after the prefetch is out
    // The partial sums of a token are added in an order that does not depend on the number of tokens
    // (SL slices whatever Tp is: with 32 tokens half of the threads sit this out), so a row's factor,
    // and with it everything computed from it, is bitwise the same in a step of 1 and of 64 rows.
    static_assert(TB <= 2, "the statistics reduction is laid out for up to 64 tokens");
    if (with_norm) {
        constexpr int C4 = Tp / 4, SL = 16;
        const int col = tid % C4, sl = tid / C4;
        const float4* sp = (const float4*)a.ssq_in + col;
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int i = sl + k * SL;
            sv[k] = (sl < SL && i < a.n_ssq) ? sp[(size_t)i * C4] : make_float4(0.f, 0.f, 0.f, 0.f);
        }
        for (int i0 = sl + 8 * SL; sl < SL && i0 < a.n_ssq; i0 += 8 * SL) {   // more than 8 rows per thread (hidden size above 256 * SL)
            float4 v[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const int i = i0 + k * SL;
                v[k] = (i < a.n_ssq) ? sp[(size_t)i * C4] : make_float4(0.f, 0.f, 0.f, 0.f);
            }
#pragma unroll
            for (int k = 0; k < 8; ++k) { s4.x += v[k].x; s4.y += v[k].y; s4.z += v[k].z; s4.w += v[k].w; }
        }
    }

    FV_TS(1)
    DPlan pl;
    pl.init(a, wg, wave);
    const int nseg = pl.nseg;
    const uint4* const zeros = a.zeros;

    // ---- request stream
    DReq rq;
    auto enter_slice = [&](int s) {     // position the stream at the first non-empty slice >= s
        rq.s = s; rq.j = 0; rq.n = 0; rq.n3 = 0; rq.wp = zeros; rq.xp = zeros;
        while (rq.s < nseg) {
            int gi, ws, we;
            pl.slice(rq.s, gi, ws, we);
            if (we > ws) {
                rq.n = we - ws; rq.n3 = (rq.n + 2) / 3 * 3;
                // weights are tiled [strip pair][half K batch][2 strips][4 frags]: a paired stage (half a batch of both
                // strips) is 8 KiB contiguous, a one-strip stage (a whole batch of one strip) two 4 KiB pieces 8 KiB apart
                rq.wp = (RS == 2) ? a.Wt + ((size_t)gi * a.NB + ws) * (FV_FRAGS * 64) + lane
                                  : a.Wt + (((size_t)(gi >> 1) * (2 * a.NB) + 2 * ws) * 2 + (gi & 1)) * (4 * 64) + lane;
                rq.xp = a.X + (size_t)ws * (2 * SF * Tp) + g * Tp + tl;
                return;
            }
            ++rq.s;
        }
    };
    // Loads are never branched around (the wait counts rely on a fixed number of loads per stage).
    // A padded stage reads from a block of zeros instead, with the same constant offsets (so the
    // offsets stay instruction immediates) but one address for all lanes: a single cache-line
    // request per instruction rather than 1 KiB, and products that add nothing.
    auto load_w = [&](uint4 (&dst)[FV_FRAGS]) {
#ifdef FV_PROBE_NO_W
        return;
#endif
        const bool live = rq.j < rq.n;
        const uint4* p = live ? rq.wp : zeros;
        // tile order inside a stage: paired: (strip r, frag f) at r*4 + f; one strip: frags 0-3, then frags 4-7 one
        // pair-row (8 tiles) further on
#pragma unroll
        for (int i = 0; i < FV_FRAGS; ++i) dst[i] = p[((RS == 2 || i < 4) ? i : i + 4) * 64];
    };
    auto load_x = [&](uint4 (&dst)[NX]) {
#ifdef FV_PROBE_NO_X
        return;
#endif
        const bool live = rq.j < rq.n;
        const uint4* p = live ? rq.xp : zeros;
#pragma unroll
        for (int f = 0; f < SF; ++f)
#pragma unroll
            for (int tb = 0; tb < TB; ++tb) dst[f * TB + tb] = p[f * (2 * Tp) + tb * 32];
    };
    auto advance = [&]() {
        ++rq.j;
        rq.wp += (RS == 2 ? FV_FRAGS : 2 * FV_FRAGS) * 64;
        rq.xp += 2 * SF * Tp;
        if (rq.j >= rq.n3) enter_slice(rq.s + 1);   // also taken, harmlessly, once the stream has ended
    };

    uint4 x[3][NX], w[3][FV_FRAGS];
    // Timing aid (stand-alone probe builds only): with FV_PROBE_NO_W / FV_PROBE_NO_X the weight / activation
    // requests are left out and the matrix instructions run on constants, which shows what a launch costs
    // apart from its operand traffic.  The results are meaningless; nothing in the library defines these.
#ifdef FV_PROBE_NO_W
    for (int i_ = 0; i_ < 3; ++i_) for (int j_ = 0; j_ < FV_FRAGS; ++j_) w[i_][j_] = make_uint4(tid, 1, 0, 0);
#endif
#ifdef FV_PROBE_NO_X
    for (int i_ = 0; i_ < 3; ++i_) for (int j_ = 0; j_ < NX; ++j_) x[i_][j_] = make_uint4(tid, 0, 0, 0);
#endif
    enter_slice(0);
    FV_TS(2)
    // prologue in the loop's own issue order: X(0) W(0) X(1) W(1) X(2) W(2)
#pragma unroll
    for (int i = 0; i < 3; ++i) {
        load_x(x[i]);
        __builtin_amdgcn_sched_barrier(0);
        load_w(w[i]);
        __builtin_amdgcn_sched_barrier(0);
        advance();
        if (i == 0) { FV_TS(3) }
    }
    FV_TS(4)

    if (with_norm) {
        constexpr int C4 = Tp / 4, SL = 16;
        const int col = tid % C4, sl = tid / C4;
#pragma unroll
        for (int k = 0; k < 8; ++k) { s4.x += sv[k].x; s4.y += sv[k].y; s4.z += sv[k].z; s4.w += sv[k].w; }
        if (sl < SL) ((float4*)red_lds)[sl * C4 + col] = s4;
        __syncthreads();
        if (tid < Tp) {
            float tot = 0.f;
#pragma unroll
            for (int p = 0; p < SL; ++p) tot += red_lds[p * Tp + tid];
            rinv_lds[tid] = rsqrtf(tot * a.inv_h + a.eps);
        }
        __syncthreads();
    }

    // One stage: multiply what register set S holds, then request into it the stage three ahead.
#define FV_DSTAGE(S)                                                                        \
    {                                                                                       \
        _Pragma("unroll") for (int r_ = 0; r_ < RS; ++r_)                                   \
        _Pragma("unroll") for (int f = 0; f < SF; ++f)                                      \
            _Pragma("unroll") for (int tb = 0; tb < TB; ++tb)                               \
                acc[r_ * TB + tb] = Tr<EL>::mma(w[S][r_ * SF + f], x[S][f * TB + tb], acc[r_ * TB + tb]); \
        __builtin_amdgcn_sched_barrier(0);                                                  \
        load_x(x[S]);                                                                       \
        __builtin_amdgcn_sched_barrier(0);                                                  \
        load_w(w[S]);                                                                       \
        __builtin_amdgcn_sched_barrier(0);                                                  \
        advance();                                                                          \
    }

    // ---- what happens to the sums of a segment
    //
    // Three wavefronts stream (they take in what the compute unit can take in: a fourth adds nothing),
    // the fourth adds up their sums at the ends of segments while they stream on: the streamers put
    // their accumulators into one of two LDS areas, meet the fourth wavefront at a barrier and start the
    // next segment; the fourth adds the three sets in wavefront order and PARKS the sum in LDS.
    // Nothing leaves the compute unit in the middle of a range: a global store (or atomic) between the
    // streaming requests costs the launch 3-6 us whichever wavefront issues it (measured: one 16-byte
    // store per lane in mid-range, any cache policy), whether it is a partial tile for another
    // workgroup or the output of a finished row group.  At the end of the range all four wavefronts
    // take one tile each: the partial tiles other workgroups wait for are stored first, then the row
    // groups this workgroup finishes get their epilogue.  (Ranges of more than FV_PARK segments -- very
    // wide matrices -- have the fourth wavefront do that for the parked segments in mid-range, once per
    // FV_PARK segments.)
    //
    // Who finishes a row group: whoever had its whole K range, else its FIRST contributor.  The ranges
    // are contiguous, so the first contributor meets the group in the last segment of its own range
    // and every other contributor in its first (segment index 0 of its partial area).
    //
    // Partial tiles cross XCDs whose L2s are not coherent: write-through stores and loads that bypass
    // the caches, 128 bits per lane through a raw buffer descriptor over the partial area (addresses
    // bounds-checked in hardware), layout per tile [4 register quads][64 lanes][4].  No
    // acknowledgement, ticket or flag: the data says itself whether it has arrived.  The partial area
    // is all zeros whenever a launch of these kernels starts; a contributor sets the lowest mantissa
    // bit of every value it stores, so a reader that finds that bit in all 16 values of all 64 lanes
    // of a tile has the whole tile, whatever order the stores landed in (every 4-byte element vouches
    // for itself).  The reader clears the bit again before it adds, so a sum does not depend on it,
    // and writes zeros back over every tile it has consumed, which leaves the area as it found it.
    float4* const park = (float4*)(red_lds + 1024 + 4);       // [FV_PARK][NT][4 quads][64 lanes]
    auto park_tile = [&](int e, int t) {                       // sums of segment e, tile t: three sets added, parked
        const float4* sums = (const float4*)red + (size_t)(e & 1) * FV_STREAMERS * NT * 256 + lane;
        float4* pk = park + ((size_t)((e % FV_PARK) * NT + t) * 4) * 64 + lane;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            float4 sum = sums[((size_t)(0 * NT + t) * 4 + q) * 64];
#pragma unroll
            for (int w_ = 1; w_ < FV_STREAMERS; ++w_) {
                const float4 v = sums[((size_t)(w_ * NT + t) * 4 + q) * 64];
                sum.x += v.x; sum.y += v.y; sum.z += v.z; sum.w += v.w;
            }
            pk[q * 64] = sum;
        }
    };
    auto flush_parked = [&](int s0, int s1, int t_lo, int t_hi) {   // segments s0..s1 (at most FV_PARK), tiles [t_lo, t_hi)
        constexpr int SC1 = 16;
        const __amdgpu_buffer_rsrc_t prs = __builtin_amdgcn_make_buffer_rsrc((void*)a.part, 0, (int)a.part_bytes, 0x00020000);
        // pass 1: what other workgroups wait for.  A segment that starts inside its row group belongs
        // to a later contributor; one that starts the group without covering it is the first
        // contributor's (the table says so also for the odd cases).
        for (int e = s0; e <= s1; ++e) {
            int gi, b0, nb;
            pl.segment(e, gi, b0, nb);
            if (nb == a.NB || (b0 == 0 && wg == a.tab_cf[gi])) continue;
            const unsigned mark = a.mark;
            for (int t = t_lo; t < t_hi; ++t) {
                const float4* pk = park + ((size_t)((e % FV_PARK) * NT + t) * 4) * 64 + lane;
                const unsigned o = ((unsigned)(wg * a.segmax * NT + t) * 1024u + (unsigned)lane * 4u) * 4u;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const float4 f = pk[q * 64];
                    u32x4 v;
                    v.x = (__float_as_uint(f.x) & ~1u) | mark;
                    v.y = (__float_as_uint(f.y) & ~1u) | mark;
                    v.z = (__float_as_uint(f.z) & ~1u) | mark;
                    v.w = (__float_as_uint(f.w) & ~1u) | mark;
                    __builtin_amdgcn_raw_buffer_store_b128(v, prs, o + q * 1024u, 0, SC1);
                }
            }
        }
        // pass 2: the row groups this workgroup finishes
        for (int e = s0; e <= s1; ++e) {
            int gi, b0, nb;
            pl.segment(e, gi, b0, nb);
            const bool whole = (nb == a.NB);
            int c_first = wg, c_last = wg;
            if (!whole) {
                if (b0 != 0) continue;
                c_first = a.tab_cf[gi]; c_last = a.tab_cl[gi];
                if (wg != c_first) continue;
            }
            for (int t = t_lo; t < t_hi; ++t) {
                auto tile_ofs = [&](int wg_) -> unsigned {
                    return ((unsigned)(wg_ * a.segmax * NT + t) * 1024u + (unsigned)lane * 4u) * 4u;
                };
                const int strip = gi * RS + t / TB, tb_ = t % TB;
                // what the residual and the rotary epilogues read besides the GEMM result is requested
                // now, so that it travels while the partial tiles are fetched
                constexpr bool resid = EPI == EPI_RESID, qkv = EPI == EPI_QKV;
                EpiPre pre;
                const bool mine_out = strip < a.n_strips;
                bool have_pre = false;
                if (resid && mine_out) { resid_preload(a, Tp, strip, tb_, lane, pre); have_pre = true; }
                if (qkv && mine_out) have_pre = rope_preload<D>(a, strip, tb_, lane, pre);
                float r[16];
                {
                    const float4* pk = park + ((size_t)((e % FV_PARK) * NT + t) * 4) * 64 + lane;
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const float4 f = pk[q * 64];
                        r[4 * q] = f.x; r[4 * q + 1] = f.y; r[4 * q + 2] = f.z; r[4 * q + 3] = f.w;
                    }
                }
                for (int c0 = c_first + 1; c0 <= c_last; c0 += 4) {   // ascending order, four tiles in flight
                    u32x4 v[4][4];
                    for (unsigned spins = 0;; ++spins) {
#pragma unroll
                        for (int k = 0; k < 4; ++k) {
                            const int c = (c0 + k <= c_last) ? c0 + k : c_last;
                            const unsigned o = tile_ofs(c);
#pragma unroll
                            for (int q = 0; q < 4; ++q) v[k][q] = __builtin_amdgcn_raw_buffer_load_b128(prs, o + q * 1024u, 0, SC1);
                        }
                        unsigned all1 = 1u;
#pragma unroll
                        for (int k = 0; k < 4; ++k)
#pragma unroll
                            for (int q = 0; q < 4; ++q) all1 &= v[k][q].x & v[k][q].y & v[k][q].z & v[k][q].w;
                        if (__all((int)(all1 & 1u))) break;
                        // Not there yet (a contributor that is still streaming).  The wait is bounded: a
                        // contributor that never delivers leaves a mark the host turns into an error.
                        if (spins >= a.spin_limit) {
                            if (lane == 0) __hip_atomic_store(a.fault, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                            break;
                        }
                        __builtin_amdgcn_s_sleep(16);
                    }
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        const float m = (c0 + k <= c_last) ? 1.f : 0.f;
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            r[4 * q] += m * __uint_as_float(v[k][q].x & ~1u);
                            r[4 * q + 1] += m * __uint_as_float(v[k][q].y & ~1u);
                            r[4 * q + 2] += m * __uint_as_float(v[k][q].z & ~1u);
                            r[4 * q + 3] += m * __uint_as_float(v[k][q].w & ~1u);
                        }
                    }
                    // the tiles just consumed go back to zero (nobody reads them again in this launch)
                    u32x4 zero4; zero4.x = 0u; zero4.y = 0u; zero4.z = 0u; zero4.w = 0u;
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        if (c0 + k > c_last) break;
                        const unsigned o = tile_ofs(c0 + k);
#pragma unroll
                        for (int q = 0; q < 4; ++q) __builtin_amdgcn_raw_buffer_store_b128(zero4, prs, o + q * 1024u, 0, SC1);
                    }
                }
                if (mine_out) gemm_epilogue<EL, D, EPI>(a, Tp, strip, tb_, lane, r, rinv_lds, pre, have_pre);
            }
        }
    };

    FV_TS(5)
    for (int s = 0; s < nseg; ++s) {
        if (wave < FV_STREAMERS) {
            int gi, ws, we;
            pl.slice(s, gi, ws, we);
            const int rounds = (we - ws + 2) / 3;
            floatx16 acc[NT];
            zero_acc<NT>(acc);
            for (int r = 0; r < rounds; ++r) {
                FV_DSTAGE(0)
                FV_DSTAGE(1)
                FV_DSTAGE(2)
            }
            // this wavefront's sums of segment s (zeros if none of its stages were ours) into LDS
            // (16 bytes per lane and access: [area][wavefront][tile][register quad][lane])
            float4* my = (float4*)red + ((size_t)(s & 1) * FV_STREAMERS + wave) * NT * 256 + lane;
#pragma unroll
            for (int t_ = 0; t_ < NT; ++t_)
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    my[(t_ * 4 + q) * 64] = make_float4(acc[t_][4 * q], acc[t_][4 * q + 1], acc[t_][4 * q + 2], acc[t_][4 * q + 3]);
            if (s == 0) { FV_TS(6) }
        }
        // The streamers arrive here with their sums in area s & 1; the fourth wavefront arrives when it
        // has parked segment s - 1, so area s & 1 (last read for segment s - 2) is free again, and what
        // it parked is visible to everybody behind this barrier.
        __syncthreads();
        const int s0 = s - s % FV_PARK;
        if (s == nseg - 1) {               // nothing left to stream: one tile each
            if (wave < NT) { park_tile(s, wave); flush_parked(s0, s, wave, wave + 1); }
        } else if (wave == FV_STREAMERS) {
            for (int t = 0; t < NT; ++t) park_tile(s, t);
            if (s % FV_PARK == FV_PARK - 1) flush_parked(s0, s, 0, NT);
        }
    }
    FV_TS(7)
#undef FV_DSTAGE
}

// Which range of the work split a workgroup takes.  Workgroups go to the 8 XCDs round-robin (workgroup b
// runs on XCD b % 8).  Where a row group is shared by three or more workgroups (few row groups, long K:
// O and down), neighbours in the split are given to workgroups of one XCD: the partial tiles then meet
// the finisher's looks in that XCD's L2 (O 15.0 -> 14.2 us, down 24.7 -> 24.4 us at the 7B shape).
// Matrices with one or two contributors per row group lose as much as they gain (each XCD then streams
// one contiguous eighth of the weights) and keep the plain order.  Only locality depends on the dispatch
// order: the exchange itself is written through and read past the caches either way.
__device__ __forceinline__ int split_index(const GemmArgs& a) {
    const int b = (int)blockIdx.x;
    if ((a.G & 7) == 0 && !a.aligned && 2 * a.NG <= a.G) return (b & 7) * (a.G >> 3) + (b >> 3);
    return b;
}

template <typename EL, int TB, int D, int EPI>
__global__ __launch_bounds__(256, 1) void k_gemm_direct(GemmArgs a) {
    extern __shared__ __attribute__((aligned(16))) float smem_dyn[];   // FV_DIRECT_SMEM_FLOATS(TB) floats
    gemm_direct_body<EL, TB, D, EPI>(a, split_index(a), smem_dyn);
}

// Two strips per wavefront, half-batch stages.  a.NG counts 64-row groups, a.NB half batches.
template <typename EL, int TB, int D, int EPI>
__global__ __launch_bounds__(256, 1) void k_gemm_paired(GemmArgs a) {
    extern __shared__ __attribute__((aligned(16))) float smem_dyn[];   // FV_PAIRED_SMEM_FLOATS(TB) floats
    gemm_direct_body<EL, TB, D, EPI, 2>(a, split_index(a), smem_dyn);
}
