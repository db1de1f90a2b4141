// Skinny GEMM for up to 64 tokens, "direct" form: one 32-row strip per workgroup at a time,
// the four wavefronts split the K range of that strip between them, and both MFMA operands
// go straight from global memory to registers (weights from HBM, activations from L2): no
// LDS and no workgroup barrier inside the streaming loop, so every wavefront runs its own
// software pipeline and drifts freely.
//
// Work split: the (strip, K batch) space is cut into G equal contiguous ranges (stream-K).
// The part of a range inside one strip is a segment; at the end of a segment the four
// wavefronts add their accumulators through LDS (fixed order).  A segment that covers the
// whole K range goes to the epilogue at once.  Otherwise the workgroup stores its partial
// tile, draws a ticket on the strip's counter, and whoever draws the last ticket sums the
// partial tiles in ascending workgroup order and runs the epilogue.  With at least one strip
// per workgroup a strip has at most three contributors, usually two, so the tail is short.
//
// Per wavefront and K batch: 8 weight tiles (1 KiB each) and 8*TB activation tiles.  Weight
// and activation tiles are requested three batches ahead into three rotating register sets, in
// a fixed issue order, so the hardware's in-order load counter lets each wait be exact.
#pragma once
// (included from fv_kernels.hpp after GemmArgs, gemm_epilogue and zero_acc)

// Shared-memory needs of the direct GEMM body, in floats: three accumulator staging slots
// [3][4 wavefronts][TB][16][64], RMSNorm factors [Tp], reduction scratch [1024], ticket.
#define FV_DIRECT_SMEM_FLOATS(TB) (3 * 4 * (TB) * 1024 + (TB) * 32 + 1024 + 4)

template <typename EL, int D, int EPI, bool COH>
__device__ __forceinline__ void epilogue_dispatch(const GemmArgs& a, int Tp, int strip, int tb, int lane, float (&r)[16],
                                                  const float* rinv_lds) {
    if constexpr (EPI >= 0) {
        gemm_epilogue<EL, D, EPI, COH>(a, Tp, strip, tb, lane, r, rinv_lds);
    } else {
        switch (a.epi) {
            case EPI_QKV: gemm_epilogue<EL, D, EPI_QKV, COH>(a, Tp, strip, tb, lane, r, rinv_lds); break;
            case EPI_RESID: gemm_epilogue<EL, D, EPI_RESID, COH>(a, Tp, strip, tb, lane, r, rinv_lds); break;
            case EPI_SWIGLU: gemm_epilogue<EL, D, EPI_SWIGLU, COH>(a, Tp, strip, tb, lane, r, rinv_lds); break;
            default: gemm_epilogue<EL, D, EPI_LOGITS, COH>(a, Tp, strip, tb, lane, r, rinv_lds); break;
        }
    }
}

// This wavefront's view of its workgroup's range of the (strip, K batch) space.
struct DCur { int s, gi, b, e, lgi, lb; };   // position in the wavefront's batch stream; (lgi, lb) = last valid
struct DPlan {
    int u0, u1, g0, nseg, NB, wave;
    __device__ __forceinline__ void init(const GemmArgs& a, int wg, int wave_) {
        // computed, not looked up: a table read would put one more memory round trip in front of
        // the first weight load
        const long long U = (long long)a.NG * a.NB;
        u0 = (int)(U * wg / a.G);
        u1 = (int)(U * (wg + 1) / a.G);
        NB = a.NB; wave = wave_;
        g0 = u0 / NB;
        nseg = 1;
        for (int e_ = (g0 + 1) * NB; e_ < u1; e_ += NB) ++nseg;
    }
    // segment s: strip gi, batches [b0, b0 + nb); this wavefront's quarter [ws, we)
    __device__ __forceinline__ void segment(int s, int& gi, int& b0, int& nb) const {
        gi = g0 + s;
        b0 = (s == 0) ? u0 - g0 * NB : 0;
        const int rem = u1 - gi * NB;
        nb = (rem < NB ? rem : NB) - b0;
    }
    __device__ __forceinline__ void slice(int s, int& gi, int& ws, int& we) const {
        int b0, nb;
        segment(s, gi, b0, nb);
        ws = b0 + nb * wave / 4;
        we = b0 + nb * (wave + 1) / 4;
    }
    __device__ __forceinline__ void settle(DCur& c) const {   // skip empty slices
        while (c.s < nseg && c.b >= c.e) {
            ++c.s;
            if (c.s < nseg) slice(c.s, c.gi, c.b, c.e);
        }
        if (c.s < nseg) { c.lgi = c.gi; c.lb = c.b; }
    }
    __device__ __forceinline__ void start(DCur& c) const {
        c.s = 0; c.lgi = g0; c.lb = u0 - g0 * NB;   // a valid address even if this wavefront has no batch at all
        slice(0, c.gi, c.b, c.e);
        settle(c);
    }
    __device__ __forceinline__ void next(DCur& c) const { if (c.s < nseg) { ++c.b; settle(c); } }
};

// Loads are never branched around (the wait counts rely on a fixed number of loads per stage).
// Past the end of the stream they all read one and the same 16 bytes instead: a single
// cache-line request per instruction rather than 1 KiB, so the filler costs next to nothing.
__device__ __forceinline__ void dload_w(uint4 (&dst)[FV_FRAGS], const uint4* __restrict__ base, int lane, int NB, const DCur& c, int nseg) {
    const bool live = c.s < nseg;
    const uint4* p = live ? base + ((size_t)c.lgi * NB + c.lb) * (FV_FRAGS * 64) + lane : base;
    const int st = live ? 64 : 0;
#pragma unroll
    for (int f = 0; f < FV_FRAGS; ++f) dst[f] = p[f * st];
}

// Issues the first three weight batches of a GEMM into `w` before the activations exist (the
// persistent kernel calls this ahead of the grid barrier that ends the previous phase).
__device__ __forceinline__ void gemm_direct_prefetch(const GemmArgs& a, int wg, uint4 (&w)[3][FV_FRAGS]) {
    if (wg >= a.G) return;
    const int lane = threadIdx.x & 63;
    DPlan pl;
    pl.init(a, wg, __builtin_amdgcn_readfirstlane(threadIdx.x >> 6));
    DCur cw;
    pl.start(cw);
    dload_w(w[0], a.Wt, lane, a.NB, cw, pl.nseg); pl.next(cw);
    dload_w(w[1], a.Wt, lane, a.NB, cw, pl.nseg); pl.next(cw);
    dload_w(w[2], a.Wt, lane, a.NB, cw, pl.nseg);
}

// EPI >= 0: epilogue fixed at compile time; EPI = -1: taken from a.epi at run time (the persistent
// step kernel runs all its GEMMs through one copy of this body).  COH: outputs are read by other
// workgroups of the same launch (see st_u64).  `wg` is this workgroup's index in the split.
// `w` are the three weight register sets; if `preloaded`, gemm_direct_prefetch already filled them.
template <typename EL, int TB, int D, int EPI, bool COH>
__device__ __forceinline__ void gemm_direct_body(const GemmArgs& a, int wg, float* smem, uint4 (&w)[3][FV_FRAGS], bool preloaded) {
    constexpr int Tp = TB * 32;
    constexpr int NX = FV_FRAGS * TB;            // activation tiles per batch
    float* red = smem;                           // [slot][wave][tb][16][64]
    float* rinv_lds = red + 3 * 4 * TB * 1024;
    float* red_lds = rinv_lds + Tp;              // 16-byte aligned: Tp is a multiple of 32
    int* ticket_lds = (int*)(red_lds + 1024);
    const bool with_norm = (EPI >= 0) ? (EPI != EPI_RESID) : (a.epi != EPI_RESID);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int tl = lane & 31, g = lane >> 5;
    if (wg >= a.G) return;

    DPlan pl;                                    // NG = strips here
    pl.init(a, wg, wave);
    const int u0 = pl.u0, u1 = pl.u1, g0 = pl.g0, nseg = pl.nseg;
    (void)u0; (void)u1; (void)g0;
    typedef DCur Cur;
    auto cur_next = [&](Cur& c) { pl.next(c); };

    auto load_w = [&](uint4 (&dst)[FV_FRAGS], const Cur& c) { dload_w(dst, a.Wt, lane, a.NB, c, nseg); };
    auto load_x = [&](uint4 (&dst)[NX], const Cur& c) {
        const bool live = c.s < nseg;   // past the end: one shared 16-byte read per instruction (see dload_w)
        const uint4* p = live ? a.X + (size_t)c.lb * (16 * Tp) + g * Tp + tl : a.X;
        const int sf = live ? 2 * Tp : 0, stb = live ? 32 : 0;
#pragma unroll
        for (int f = 0; f < FV_FRAGS; ++f)
#pragma unroll
            for (int tb = 0; tb < TB; ++tb) dst[f * TB + tb] = p[f * sf + tb * stb];
    };

    float4 s4 = make_float4(0.f, 0.f, 0.f, 0.f);
    if (with_norm) {
        // RMSNorm factor of every token from the [n_ssq][Tp] partial sums of squares: the loads go
        // out first (L2 hits), the weight/activation prefetch right behind them, the reduction after
        constexpr int C4 = Tp / 4, SL = 256 / C4;
        const int col = tid % C4, sl = tid / C4;
        const float4* sp = (const float4*)a.ssq_in + col;
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
    }
    uint4 x[3][NX];
    Cur cc, cx, cw;          // compute cursor; activation- and weight-prefetch cursors (3 batches ahead)
    pl.start(cc);
    cx = cc; cw = cc;
    if (preloaded) {
        // the weights of batches 0..2 are already on their way: only the activations are missing
        load_x(x[0], cx); cur_next(cx);
        load_x(x[1], cx); cur_next(cx);
        load_x(x[2], cx); cur_next(cx);
        cur_next(cw); cur_next(cw); cur_next(cw);
    } else {
        // prologue in the loop's own issue order: X(0) W(0) X(1) W(1) X(2) W(2)
        load_x(x[0], cx); cur_next(cx);
        __builtin_amdgcn_sched_barrier(0);
        load_w(w[0], cw); cur_next(cw);
        __builtin_amdgcn_sched_barrier(0);
        load_x(x[1], cx); cur_next(cx);
        __builtin_amdgcn_sched_barrier(0);
        load_w(w[1], cw); cur_next(cw);
        __builtin_amdgcn_sched_barrier(0);
        load_x(x[2], cx); cur_next(cx);
        __builtin_amdgcn_sched_barrier(0);
        load_w(w[2], cw); cur_next(cw);
    }
    __builtin_amdgcn_sched_barrier(0);

    if (with_norm) {
        constexpr int C4 = Tp / 4, SL = 256 / C4;
        const int col = tid % C4, sl = tid / C4;
        ((float4*)red_lds)[sl * C4 + col] = s4;
        __syncthreads();
        if (tid < Tp) {
            float tot = 0.f;
#pragma unroll
            for (int p = 0; p < SL; ++p) tot += red_lds[p * Tp + tid];
            rinv_lds[tid] = rsqrtf(tot * a.inv_h + a.eps);
        }
        __syncthreads();
    }
    floatx16 acc[TB];
    zero_acc<TB>(acc);
    int fs = 0;             // next segment to finish (workgroup-wide, in order)
    int acc_seg = cc.s;     // segment the accumulators belong to
    unsigned staged = 0;    // bit (s - fs): this wavefront has put real sums for segment s into its slot

    // A wavefront that has done its last batch of a segment parks its accumulators in LDS slot
    // (segment % 3) at once -- short code, repeated in each of the three pipeline stages -- and
    // streams on.  The heavy part (sum over wavefronts, partial exchange, epilogue) sits in one
    // place, at the bottom of the loop.  A wavefront parks at most three segments per round and
    // finishes all of them at the bottom, so three slots are enough.
    auto park = [&]() {
        float* slot = red + (size_t)((acc_seg % 3) * 4 + wave) * TB * 1024 + lane;
#pragma unroll
        for (int tb = 0; tb < TB; ++tb)
#pragma unroll
            for (int i = 0; i < 16; ++i) slot[(tb * 16 + i) * 64] = acc[tb][i];
        zero_acc<TB>(acc);
        staged |= 1u << (acc_seg - fs);
    };

    // end of segment s for the whole workgroup
    auto finish_segment = [&](int s) {
        int gi, b0, nb;
        pl.segment(s, gi, b0, nb);
        float* slot0 = red + (size_t)((s % 3) * 4) * TB * 1024 + lane;
        if (!(staged & 1u)) {   // no batch of this segment was ours: contribute zeros
#pragma unroll
            for (int j = 0; j < TB * 16; ++j) slot0[((size_t)wave * TB * 16 + j) * 64] = 0.f;
        }
        staged >>= 1;
        __syncthreads();
        float r[16];
        if (wave < TB) {   // wavefront tb sums tile tb over the four wavefronts, in wavefront order
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                float sum = slot0[((size_t)(0 * TB + wave) * 16 + i) * 64];
#pragma unroll
                for (int w_ = 1; w_ < 4; ++w_) sum += slot0[((size_t)(w_ * TB + wave) * 16 + i) * 64];
                r[i] = sum;
            }
        }
        bool finish = (nb == a.NB);   // the whole K range was ours: straight to the epilogue
        if (!finish) {
            // partial tile out with agent-scope atomic stores (write-through: partials and tickets
            // cross XCDs whose L2s are not coherent), acknowledged before the ticket is drawn
            if (wave < TB) {
                float* pp = a.part + (((size_t)wg * a.segmax + s) * TB + wave) * 1024 + lane;
#pragma unroll
                for (int i = 0; i < 16; ++i) __hip_atomic_store(pp + i * 64, r[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            const int c_first = a.tab_cf[gi], c_last = a.tab_cl[gi];
            __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): stores count in vmcnt on this target
            __syncthreads();
            if (tid == 0) *ticket_lds = __hip_atomic_fetch_add(&a.tickets[gi], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __syncthreads();
            if (*ticket_lds == c_last - c_first) {
                finish = true;
                if (tid == 0) __hip_atomic_store(&a.tickets[gi], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // for the next launch
                if (wave < TB) {
#pragma unroll
                    for (int i = 0; i < 16; ++i) r[i] = 0.f;
                    for (int c0 = c_first; c0 <= c_last; c0 += 2) {   // ascending order, two tiles in flight
                        float v[2][16];
#pragma unroll
                        for (int k = 0; k < 2; ++k) {
                            const int c = (c0 + k <= c_last) ? c0 + k : c_last;
                            const int cseg = gi - a.tab_g0[c];
                            const float* cp = a.part + (((size_t)c * a.segmax + cseg) * TB + wave) * 1024 + lane;
#pragma unroll
                            for (int i = 0; i < 16; ++i) v[k][i] = __hip_atomic_load(cp + i * 64, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        }
#pragma unroll
                        for (int k = 0; k < 2; ++k) {
                            const float m = (c0 + k <= c_last) ? 1.f : 0.f;
#pragma unroll
                            for (int i = 0; i < 16; ++i) r[i] += m * v[k][i];
                        }
                    }
                }
            }
        }
        if (finish && wave < TB) epilogue_dispatch<EL, D, EPI, COH>(a, Tp, gi, wave, lane, r, rinv_lds);
        __syncthreads();   // the slot and ticket_lds are reused
    };

#define FV_DSTAGE(S)                                                                        \
    {                                                                                       \
        if (cc.s < nseg) {                                                                  \
            _Pragma("unroll") for (int f = 0; f < FV_FRAGS; ++f)                            \
                _Pragma("unroll") for (int tb = 0; tb < TB; ++tb)                           \
                    acc[tb] = Tr<EL>::mma(w[S][f], x[S][f * TB + tb], acc[tb]);             \
        }                                                                                   \
        __builtin_amdgcn_sched_barrier(0);                                                  \
        load_x(x[S], cx); cur_next(cx);                                                     \
        __builtin_amdgcn_sched_barrier(0);                                                  \
        load_w(w[S], cw); cur_next(cw);                                                     \
        __builtin_amdgcn_sched_barrier(0);                                                  \
        cur_next(cc);                                                                       \
        if (cc.s != acc_seg) { park(); acc_seg = cc.s; }                                    \
    }

    for (;;) {
        while (fs < cc.s) { finish_segment(fs); ++fs; }   // the only place the heavy code is instantiated
        if (fs >= nseg) break;
        FV_DSTAGE(0)
        FV_DSTAGE(1)
        FV_DSTAGE(2)
    }
#undef FV_DSTAGE
}

template <typename EL, int TB, int D, int EPI>
__global__ __launch_bounds__(256, 1) void k_gemm_direct(GemmArgs a) {
    extern __shared__ __attribute__((aligned(16))) float smem_dyn[];   // FV_DIRECT_SMEM_FLOATS(TB) floats
    uint4 w[3][FV_FRAGS];
    gemm_direct_body<EL, TB, D, EPI, false>(a, blockIdx.x, smem_dyn, w, false);
}
