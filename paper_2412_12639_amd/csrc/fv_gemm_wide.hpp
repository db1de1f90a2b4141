// Skinny GEMM for up to 64 tokens, "wide" form, for the matrices with many output rows (QKV,
// gate/up, LM head).  An experiment kept as an option (FV_GEMM=wide): the vector-load path of a
// compute unit is a shared resource between weight tiles (HBM) and activation tiles (L2/L1), so
// the fewer activation bytes per weight byte the better.  Here every wavefront owns FOUR 32-row strips (a "super-strip")
// and one quarter of their K range: an activation tile (2 KiB at 64 tokens) is loaded once and
// meets four weight tiles (4 KiB), all in registers -- no LDS and no barrier in the stream.
//
// Work split as in the direct form: the (super-strip, K batch) space is cut into G equal ranges;
// the part of a range inside one super-strip is a segment; the four wavefronts of a workgroup
// split a segment's batches.  At a segment end they add their accumulators through LDS; a segment
// that covers the whole K range goes to the epilogue, otherwise partial tiles + ticket, and the
// last arriver sums in ascending workgroup order (deterministic).
//
// A wavefront moves 32 KiB of weights per batch: a strip's register set is refilled with the next
// batch's tile right after it has been multiplied (four sets, one per strip), and the single
// activation set is refilled after the batch's last product.  Only one batch ahead fits the
// register file, which exposes two memory latencies per batch; measured, this form loses to the
// paired form of the direct kernel on every matrix but the LM head.
#pragma once
// (included from fv_kernels.hpp after fv_gemm_direct.hpp)

#define FV_WS 4   // strips per wavefront
// LDS: accumulator exchange [4 wavefronts][4 strips][TB][16][64], RMSNorm factors, scratch, ticket
#define FV_WIDE_SMEM_FLOATS(TB) (4 * FV_WS * (TB) * 1024 + (TB) * 32 + 1024 + 4)

// Sum of the contributors' partial tiles (super-strip ss, strip r, token block tb) in ascending
// workgroup order, four contributions (64 loads per lane) in flight at a time; agent-scope atomic
// loads, which do not hit stale cache lines.
template <int TB>
__device__ __forceinline__ void wide_sum_partials(const GemmArgs& a, int ss, int r, int tb, int lane, int c_first, int c_last, float (&rr)[16]) {
#pragma unroll
    for (int i = 0; i < 16; ++i) rr[i] = 0.f;
    for (int c0 = c_first; c0 <= c_last; c0 += 4) {
        float v[4][16];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int c = (c0 + k <= c_last) ? c0 + k : c_last;
            const int cseg = ss - a.tab_g0[c];
            const float* cp = a.part + ((((size_t)c * a.segmax + cseg) * FV_WS + r) * TB + tb) * 1024 + lane;
#pragma unroll
            for (int i = 0; i < 16; ++i) v[k][i] = __hip_atomic_load(cp + i * 64, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const float m = (c0 + k <= c_last) ? 1.f : 0.f;
#pragma unroll
            for (int i = 0; i < 16; ++i) rr[i] += m * v[k][i];
        }
    }
}

template <typename EL, int TB, int D, int EPI, bool COH>
__device__ __forceinline__ void gemm_wide_body(const GemmArgs& a, int wg, float* smem) {
    constexpr int Tp = TB * 32;
    constexpr int NX = FV_FRAGS * TB;
    float* red = smem;                                   // [wave][strip][tb][16][64]
    float* rinv_lds = red + 4 * FV_WS * TB * 1024;
    float* red_lds = rinv_lds + Tp;
    int* ticket_lds = (int*)(red_lds + 1024);
    const bool with_norm = (EPI >= 0) ? (EPI != EPI_RESID) : (a.epi != EPI_RESID);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int tl = lane & 31, g = lane >> 5;
    if (wg >= a.G) return;

    DPlan pl;            // NG = super-strips here
    pl.init(a, wg, wave);
    const int nseg = pl.nseg;

    // weight tiles of batch (ss, b) for strip r of the super-strip; past the end of the stream all
    // lanes read one and the same 16 bytes (the loads are never branched around)
    auto load_w = [&](uint4 (&dst)[FV_FRAGS], const DCur& c, int r) {
        const bool live = c.s < nseg;
        const uint4* p = live ? a.Wt + (((size_t)c.lgi * FV_WS + r) * a.NB + c.lb) * (FV_FRAGS * 64) + lane : a.Wt;
        const int st = live ? 64 : 0;
#pragma unroll
        for (int f = 0; f < FV_FRAGS; ++f) dst[f] = p[f * st];
    };
    auto load_x = [&](uint4 (&dst)[NX], const DCur& c) {
        const bool live = c.s < nseg;
        const uint4* p = live ? a.X + (size_t)c.lb * (16 * Tp) + g * Tp + tl : a.X;
        const int sf = live ? 2 * Tp : 0, stb = live ? 32 : 0;
#pragma unroll
        for (int f = 0; f < FV_FRAGS; ++f)
#pragma unroll
            for (int tb = 0; tb < TB; ++tb) dst[f * TB + tb] = p[f * sf + tb * stb];
    };

    float4 s4 = make_float4(0.f, 0.f, 0.f, 0.f);
    if (with_norm) {   // RMSNorm statistics first (L2 hits), the stream right behind them
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

    uint4 w[FV_WS][FV_FRAGS], x[NX];
    DCur cc, cn;                 // batch being multiplied; batch being requested (one ahead)
    pl.start(cc);
    cn = cc;
    load_x(x, cn);
#pragma unroll
    for (int r = 0; r < FV_WS; ++r) load_w(w[r], cn, r);
    pl.next(cn);
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

    floatx16 acc[FV_WS][TB];
#pragma unroll
    for (int r = 0; r < FV_WS; ++r) zero_acc<TB>(acc[r]);
    int fs = 0;
    bool mine = false;   // the accumulators hold sums of segment fs

    // end of segment s for the whole workgroup: wavefront w finishes strip w of the super-strip
    auto finish_segment = [&](int s) {
        int ss, b0, nb;
        pl.segment(s, ss, b0, nb);
        float* my = red + (size_t)wave * FV_WS * TB * 1024 + lane;
#pragma unroll
        for (int r = 0; r < FV_WS; ++r)
#pragma unroll
            for (int tb = 0; tb < TB; ++tb)
#pragma unroll
                for (int i = 0; i < 16; ++i) my[((r * TB + tb) * 16 + i) * 64] = mine ? acc[r][tb][i] : 0.f;
#pragma unroll
        for (int r = 0; r < FV_WS; ++r) zero_acc<TB>(acc[r]);
        mine = false;
        __syncthreads();
        const int strip = ss * FV_WS + wave;
        const bool whole = (nb == a.NB);
        // partial tiles go out with agent-scope atomic stores (write-through across XCDs)
        float* pp = a.part + ((((size_t)wg * a.segmax + s) * FV_WS + wave) * TB) * 1024 + lane;
#pragma unroll
        for (int tb = 0; tb < TB; ++tb) {
            float rr[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                float sum = 0.f;
#pragma unroll
                for (int w_ = 0; w_ < 4; ++w_) sum += red[(((size_t)(w_ * FV_WS + wave) * TB + tb) * 16 + i) * 64 + lane];
                rr[i] = sum;
            }
            if (whole) {
                if (strip < a.n_strips) epilogue_dispatch<EL, D, EPI, COH>(a, Tp, strip, tb, lane, rr, rinv_lds, ResidPre(), false);
            } else {
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    __hip_atomic_store(pp + (tb * 16 + i) * 64, rr[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
        if (!whole) {
            // stores acknowledged, then the ticket of this super-strip; the last arriver finishes it
            const int c_first = a.tab_cf[ss], c_last = a.tab_cl[ss];
            __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
            __syncthreads();
            if (tid == 0) *ticket_lds = __hip_atomic_fetch_add(&a.tickets[ss], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __syncthreads();
            if (*ticket_lds == c_last - c_first) {
                if (tid == 0) __hip_atomic_store(&a.tickets[ss], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (strip < a.n_strips) {
#pragma unroll 1
                    for (int tb = 0; tb < TB; ++tb) {
                        float rr[16];
                        wide_sum_partials<TB>(a, ss, wave, tb, lane, c_first, c_last, rr);
                        epilogue_dispatch<EL, D, EPI, COH>(a, Tp, strip, tb, lane, rr, rinv_lds, ResidPre(), false);
                    }
                }
            }
        }
        __syncthreads();
    };

    // one batch: four strips against the same activation tiles.  Request order W0 W1 W2 X W3, so
    // that the wait for the activations at the top of the next batch leaves W3 in flight.
    for (;;) {
        while (fs < cc.s) { finish_segment(fs); ++fs; }
        if (fs >= nseg) break;
#pragma unroll
        for (int r = 0; r < FV_WS; ++r) {
#pragma unroll
            for (int f = 0; f < FV_FRAGS; ++f)
#pragma unroll
                for (int tb = 0; tb < TB; ++tb) acc[r][tb] = Tr<EL>::mma(w[r][f], x[f * TB + tb], acc[r][tb]);
            __builtin_amdgcn_sched_barrier(0);
            if (r == FV_WS - 1) load_x(x, cn);
            load_w(w[r], cn, r);
            __builtin_amdgcn_sched_barrier(0);
        }
        mine = true;
        pl.next(cn);
        pl.next(cc);
    }
}

template <typename EL, int TB, int D, int EPI>
__global__ __launch_bounds__(256, 1) void k_gemm_wide(GemmArgs a) {
    extern __shared__ __attribute__((aligned(16))) float smem_dyn[];   // FV_WIDE_SMEM_FLOATS(TB) floats
    gemm_wide_body<EL, TB, D, EPI, false>(a, blockIdx.x, smem_dyn);
}
