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

#ifndef FV_TSTAMP
#define FV_TSTAMP(k)
#endif

template <typename EL, int TB, int D, int EPI>
__global__ __launch_bounds__(256, 1) void k_gemm_direct(GemmArgs a) {
    constexpr int Tp = TB * 32;
    constexpr int NX = FV_FRAGS * TB;            // activation tiles per batch
    __shared__ float red[4 * TB * 1024];         // [wave][tb][16][64]
    __shared__ float rinv_lds[Tp];
    __shared__ __attribute__((aligned(16))) float red_lds[(EPI == EPI_RESID) ? 4 : 1024];
    __shared__ int ticket_lds;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int tl = lane & 31, g = lane >> 5;
    if ((int)blockIdx.x >= a.G) return;
    FV_TSTAMP(0)

    // NG = strips here.  The range is computed, not looked up: a table read would put one more
    // memory round trip in front of the first weight load.
    const long long U = (long long)a.NG * a.NB;
    const int u0 = (int)(U * blockIdx.x / a.G);
    const int u1 = (int)(U * (blockIdx.x + 1) / a.G);
    const int g0 = u0 / a.NB;
    int nseg = 1;
    for (int e_ = (g0 + 1) * a.NB; e_ < u1; e_ += a.NB) ++nseg;

    // this wavefront's slice [ws, we) of segment s
    auto slice = [&](int s, int& gi, int& ws, int& we) {
        gi = g0 + s;
        const int b0 = (s == 0) ? u0 - g0 * a.NB : 0;
        const int rem = u1 - gi * a.NB;
        const int e = rem < a.NB ? rem : a.NB;
        const int nb = e - b0;
        ws = b0 + nb * wave / 4;
        we = b0 + nb * (wave + 1) / 4;
    };
    struct Cur { int s, gi, b, e, lgi, lb; };   // position in this wavefront's batch stream; (lgi, lb) = last valid
    auto cur_settle = [&](Cur& c) {              // skip empty slices
        while (c.s < nseg && c.b >= c.e) {
            ++c.s;
            if (c.s < nseg) slice(c.s, c.gi, c.b, c.e);
        }
        if (c.s < nseg) { c.lgi = c.gi; c.lb = c.b; }
    };
    auto cur_init = [&](Cur& c) {
        c.s = 0; c.lgi = g0; c.lb = u0 - g0 * a.NB;   // a valid address even if this wavefront has no batch at all
        slice(0, c.gi, c.b, c.e);
        cur_settle(c);
    };
    auto cur_next = [&](Cur& c) { if (c.s < nseg) { ++c.b; cur_settle(c); } };

    const uint4* __restrict__ wl = a.Wt + lane;
    const uint4* __restrict__ xl = a.X + g * Tp + tl;
    auto load_w = [&](uint4 (&dst)[FV_FRAGS], const Cur& c) {
        const uint4* p = wl + ((size_t)c.lgi * a.NB + c.lb) * (FV_FRAGS * 64);
#pragma unroll
        for (int f = 0; f < FV_FRAGS; ++f) dst[f] = p[f * 64];
    };
    auto load_x = [&](uint4 (&dst)[NX], const Cur& c) {
        const uint4* p = xl + (size_t)c.lb * (16 * Tp);
#pragma unroll
        for (int f = 0; f < FV_FRAGS; ++f)
#pragma unroll
            for (int tb = 0; tb < TB; ++tb) dst[f * TB + tb] = p[(2 * f) * Tp + tb * 32];
    };

    float4 s4 = make_float4(0.f, 0.f, 0.f, 0.f);
    if constexpr (EPI != EPI_RESID) {
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
    uint4 w[3][FV_FRAGS], x[3][NX];
    Cur cc, cx, cw;          // compute cursor; activation- and weight-prefetch cursors (3 batches ahead)
    cur_init(cc);
    cx = cc; cw = cc;
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
    __builtin_amdgcn_sched_barrier(0);

    if constexpr (EPI != EPI_RESID) {
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
    FV_TSTAMP(1)
    floatx16 acc[TB];
    zero_acc<TB>(acc);
    int fs = 0;   // next segment to flush

    // end of segment s for the whole workgroup
    auto flush = [&](int s) {
        if (s == nseg - 1) { FV_TSTAMP(2) }
        int gi, ws, we;
        slice(s, gi, ws, we);
        const int b0 = (s == 0) ? u0 - g0 * a.NB : 0;
        const int rem = u1 - gi * a.NB;
        const int nb = (rem < a.NB ? rem : a.NB) - b0;
        // the four wavefronts' accumulators -> LDS; wavefront tb sums tile tb in wavefront order
#pragma unroll
        for (int tb = 0; tb < TB; ++tb)
#pragma unroll
            for (int i = 0; i < 16; ++i) red[((wave * TB + tb) * 16 + i) * 64 + lane] = acc[tb][i];
        zero_acc<TB>(acc);
        __syncthreads();
        float r[16];
        if (wave < TB) {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                float sum = red[((0 * TB + wave) * 16 + i) * 64 + lane];
#pragma unroll
                for (int w_ = 1; w_ < 4; ++w_) sum += red[((w_ * TB + wave) * 16 + i) * 64 + lane];
                r[i] = sum;
            }
        }
        bool finish = (nb == a.NB);   // the whole K range was ours: straight to the epilogue
        if (!finish) {
            // partial tile out with agent-scope atomic stores (write-through: partials and tickets
            // cross XCDs whose L2s are not coherent), acknowledged before the ticket is drawn
            if (wave < TB) {
                float* pp = a.part + (((size_t)blockIdx.x * a.segmax + s) * TB + wave) * 1024 + lane;
#pragma unroll
                for (int i = 0; i < 16; ++i) __hip_atomic_store(pp + i * 64, r[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            const int c_first = a.tab_cf[gi], c_last = a.tab_cl[gi];
            __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): stores count in vmcnt on this target
            __syncthreads();
            if (tid == 0) ticket_lds = __hip_atomic_fetch_add(&a.tickets[gi], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __syncthreads();
            if (ticket_lds == c_last - c_first) {
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
        if (finish && wave < TB) gemm_epilogue<EL, D, EPI>(a, Tp, gi, wave, lane, r, rinv_lds);
        __syncthreads();   // red[] and ticket_lds are reused by the next segment
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
        while (fs < cc.s) { flush(fs); ++fs; }                                              \
    }

    while (fs < cc.s) { flush(fs); ++fs; }   // leading segments in which this wavefront has no batch
    while (fs < nseg) {
        FV_DSTAGE(0)
        FV_DSTAGE(1)
        FV_DSTAGE(2)
    }
#undef FV_DSTAGE
    FV_TSTAMP(3)
}
