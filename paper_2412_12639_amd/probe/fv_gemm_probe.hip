// Stand-alone timing of the library's own weight-streaming GEMM kernel (k_gemm_paired, 64 tokens, or 32 with -DFV_PROBE_TB=1) on the
// projection shapes of a decoder layer, outside the library's step: what a launch costs when nothing
// runs (empty kernel), what the same bytes cost as a pure streaming read, what the GEMM costs per
// matrix and per layer, and -- in the build with -DFV_PROBE_STAMPS -- where inside a launch the time
// goes (one time stamp per wavefront at eight points of the kernel, through the kernel's FV_TS hook).
// Builds with -DFV_PROBE_NO_X and/or -DFV_PROBE_NO_W take the activation / weight requests out of the
// kernel's streaming loop (hooks in fv_gemm_direct.hpp): what is left is what a launch costs apart
// from its operand traffic.
//
// Weights are rotated through 3 GiB of zeros so that every launch streams HBM-cold memory; the
// arithmetic is that of the product kernel, the values are irrelevant to the timing.
//
//   fv_gemm_probe [hidden ffn q_heads kv_heads head_dim vocab]      (default: 4096 11008 32 32 128 32000)
//
// A measuring aid: nothing in the library, the tests or bench.py uses it.
#include <hip/hip_runtime.h>
#ifdef FV_PROBE_STAMPS
// one slot of 16 stamps per wavefront; written by lane 0 with a plain store
__device__ long long* g_ts;
#define FV_TS(k) if ((threadIdx.x & 63) == 0) g_ts[(blockIdx.x * 4 + (threadIdx.x >> 6)) * 16 + (k)] = wall_clock64();
#endif
#include "../csrc/fv_kernels.hpp"
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); exit(1); } } while (0)
static size_t rup(size_t x, size_t m) { return (x + m - 1) / m * m; }

// The split the library's host code makes for the paired kernel: row groups of two 32-row strips,
// K stages of 64 columns, G equal ranges of the (row group, stage) space, or whole groups per workgroup.
struct Split { int NG, NB, G, segmax, n_strips, aligned; std::vector<int> tab; int* dtab; size_t tiled; };
static Split make_split(int n_strips, int K, int nwg, int aligned) {
    Split p; p.n_strips = n_strips; p.NB = (int)rup(K, 128) / 64; p.NG = (int)rup(n_strips, FV_R) / 2; p.aligned = aligned;
    const long long U = (long long)p.NG * p.NB;
    p.G = (int)(U < nwg ? U : nwg);
    const long long per = (U + p.G - 1) / p.G;
    p.segmax = aligned ? (p.NG + p.G - 1) / p.G + 1 : (int)((per + p.NB - 1) / p.NB) + 1;
    const int G = p.G, NG = p.NG, NB = p.NB;
    p.tab.assign((size_t)2 * G + 1 + 2 * NG, 0);
    int* u0 = p.tab.data(); int* g0 = u0 + G + 1; int* cf = g0 + G; int* cl = cf + NG;
    for (int w = 0; w <= G; ++w) u0[w] = aligned ? (int)((long long)NG * w / G) * NB : (int)(U * w / G);
    for (int w = 0; w < G; ++w) g0[w] = u0[w] / NB;
    for (int gi = 0; gi < NG; ++gi) { cf[gi] = G; cl[gi] = -1; }
    for (int w = 0; w < G; ++w)
        for (int gi = g0[w]; gi <= (u0[w + 1] - 1) / NB; ++gi) { if (w < cf[gi]) cf[gi] = w; if (w > cl[gi]) cl[gi] = w; }
    CK(hipMalloc(&p.dtab, p.tab.size() * 4));
    CK(hipMemcpy(p.dtab, p.tab.data(), p.tab.size() * 4, hipMemcpyHostToDevice));
    p.tiled = (size_t)rup(n_strips, FV_R) * (rup(K, 128) / 128) * 8192;
    return p;
}

__global__ __launch_bounds__(256, 1) void k_empty(GemmArgs a) { if (a.G < 0) a.tickets[0] = 1; }

// Pure streaming read in the GEMM's launch shape: each workgroup a contiguous chunk, a quarter per
// wavefront, sixteen 1 KiB requests per wavefront in flight.
__global__ __launch_bounds__(256, 1) void k_read(const uint4* p, size_t n16, uint4* sink) {
    const size_t per_wg = n16 / gridDim.x, per_wave = per_wg / 4;
    const uint4* q = p + (size_t)blockIdx.x * per_wg + (threadIdx.x >> 6) * per_wave + (threadIdx.x & 63);
    uint4 acc = make_uint4(0, 0, 0, 0);
    const size_t iters = per_wave / (64 * 16);
    for (size_t i = 0; i < iters; ++i) {
        uint4 v[16];
#pragma unroll
        for (int k = 0; k < 16; ++k) v[k] = q[(i * 16 + k) * 64];
#pragma unroll
        for (int k = 0; k < 16; ++k) { acc.x ^= v[k].x; acc.y ^= v[k].y; acc.z ^= v[k].z; acc.w ^= v[k].w; }
    }
    if (acc.x == 0x12345678u) sink[threadIdx.x] = acc;
}

// The same loop over a small region that every workgroup reads `passes` times: after the first pass the lines
// come from the XCD's L2 (what the activation operand does in the GEMM).
__global__ __launch_bounds__(256, 1) void k_reread(const uint4* p, size_t n16, int passes, uint4* sink) {
    const size_t per_wave = n16 / 4;
    const uint4* q = p + (threadIdx.x >> 6) * per_wave + (threadIdx.x & 63);
    uint4 acc = make_uint4(0, 0, 0, 0);
    const size_t iters = per_wave / (64 * 16);
    for (int r = 0; r < passes; ++r)
        for (size_t i = 0; i < iters; ++i) {
            uint4 v[16];
#pragma unroll
            for (int k = 0; k < 16; ++k) v[k] = q[(i * 16 + k) * 64];
#pragma unroll
            for (int k = 0; k < 16; ++k) { acc.x ^= v[k].x; acc.y ^= v[k].y; acc.z ^= v[k].z; acc.w ^= v[k].w; }
        }
    if (acc.x == 0x12345678u) sink[threadIdx.x] = acc;
}

#ifndef FV_PROBE_TB
#define FV_PROBE_TB 2   // 32-token blocks per step: 2 = 64 tokens (the benchmark's tree), 1 = 32 tokens
#endif
static hipStream_t g_stream = nullptr;   // the null stream, except for the graph comparison at the end
template <int EPI> static void launch(const GemmArgs& ga) {
    hipLaunchKernelGGL((k_gemm_paired<BF16, FV_PROBE_TB, 128, EPI>), dim3(ga.G), dim3(256), FV_PAIRED_SMEM_FLOATS(FV_PROBE_TB) * 4, g_stream, ga);
}
static void launch_epi(int epi, const GemmArgs& ga) {
    switch (epi) {
        case EPI_QKV: launch<EPI_QKV>(ga); break;
        case EPI_RESID: launch<EPI_RESID>(ga); break;
        case EPI_SWIGLU: launch<EPI_SWIGLU>(ga); break;
        default: launch<EPI_LOGITS>(ga);
    }
}

int main(int argc, char** argv) {
    const int h = argc > 6 ? atoi(argv[1]) : 4096, F = argc > 6 ? atoi(argv[2]) : 11008, Hq = argc > 6 ? atoi(argv[3]) : 32,
              Hkv = argc > 6 ? atoi(argv[4]) : 32, D = argc > 6 ? atoi(argv[5]) : 128, V = argc > 6 ? atoi(argv[6]) : 32000;
    const int T = 32 * FV_PROBE_TB, Tp = 32 * FV_PROBE_TB, nwg = 256, S_pad = 1024;
    if (D != 128 || h % 128 || F % 64 || Hq % Hkv || h != Hq * D) { printf("unsupported shape\n"); return 2; }
    const size_t wbytes = (size_t)3 << 30;
    char* W; CK(hipMalloc(&W, wbytes)); CK(hipMemset(W, 0, wbytes));
    const size_t xbytes = (size_t)(F > h ? F : h) * Tp * 2 + (1 << 20);
    char* X; CK(hipMalloc(&X, xbytes)); CK(hipMemset(X, 0, xbytes));
    float* part; CK(hipMalloc(&part, (size_t)64 << 20)); CK(hipMemset(part, 0, (size_t)64 << 20));
    int* tickets; CK(hipMalloc(&tickets, 8192 * 4)); CK(hipMemset(tickets, 0, 8192 * 4));
    float* ssq; CK(hipMalloc(&ssq, 1024 * 64 * 4)); CK(hipMemset(ssq, 0, 1024 * 64 * 4));
    float* x; CK(hipMalloc(&x, (size_t)h * Tp * 4)); CK(hipMemset(x, 0, (size_t)h * Tp * 4));
    char* out; CK(hipMalloc(&out, (size_t)64 << 20)); CK(hipMemset(out, 0, (size_t)64 << 20));
    char* zb; CK(hipMalloc(&zb, 32768)); CK(hipMemset(zb, 0, 32768));
    float* gain; CK(hipMalloc(&gain, h * 4)); CK(hipMemset(gain, 0, h * 4));
    float2* rope; CK(hipMalloc(&rope, 256 * 64 * 8)); CK(hipMemset(rope, 0, 256 * 64 * 8));
    char* kv; CK(hipMalloc(&kv, (size_t)Hkv * S_pad * D * 2 * 2)); CK(hipMemset(kv, 0, (size_t)Hkv * S_pad * D * 2 * 2));

    struct Case { const char* name; int epi; Split p; size_t bytes; };
    std::vector<Case> cases = {
        {"QKV", EPI_QKV, make_split((Hq + 2 * Hkv) * D / 32, h, nwg, 0), (size_t)(Hq + 2 * Hkv) * D * h * 2},
        {"O", EPI_RESID, make_split(h / 32, Hq * D, nwg, 0), (size_t)h * Hq * D * 2},
        {"gate/up", EPI_SWIGLU, make_split(F / 16, h, nwg, 0), (size_t)2 * F * h * 2},
        {"down", EPI_RESID, make_split(h / 32, F, nwg, 0), (size_t)h * F * 2},
        {"head", EPI_LOGITS, make_split((V + 31) / 32, h, nwg, 1), (size_t)V * h * 2},
    };
    for (auto& c : cases)
        if ((size_t)c.p.G * c.p.segmax * 4 * 4096 > ((size_t)64 << 20) || c.p.NG > 8192) { printf("shape too large for the probe's buffers\n"); return 2; }
    const void* fns[4] = {(const void*)k_gemm_paired<BF16, FV_PROBE_TB, 128, EPI_QKV>, (const void*)k_gemm_paired<BF16, FV_PROBE_TB, 128, EPI_RESID>,
                          (const void*)k_gemm_paired<BF16, FV_PROBE_TB, 128, EPI_SWIGLU>, (const void*)k_gemm_paired<BF16, FV_PROBE_TB, 128, EPI_LOGITS>};
    for (const void* f : fns) CK(hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, FV_PAIRED_SMEM_FLOATS(FV_PROBE_TB) * 4));
    hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
#ifdef FV_PROBE_STAMPS
    long long* dts; CK(hipMalloc(&dts, 1024 * 16 * 8)); CK(hipMemcpyToSymbol(HIP_SYMBOL(g_ts), &dts, sizeof(dts)));
#endif
    size_t woff = 0;
    unsigned* fault; CK(hipMalloc(&fault, 256)); CK(hipMemset(fault, 0, 256));
    auto args_of = [&](Case& c) {
        GemmArgs ga; std::memset(&ga, 0, sizeof(ga));
        ga.X = (const uint4*)X; ga.part = part; ga.part_bytes = 64u << 20; ga.tickets = tickets; ga.zeros = (const uint4*)zb; ga.aligned = c.p.aligned;
        ga.NG = c.p.NG; ga.NB = c.p.NB; ga.G = c.p.G; ga.segmax = c.p.segmax; ga.T = T; ga.n_strips = c.p.n_strips;
        ga.tab_u0 = c.p.dtab; ga.tab_g0 = c.p.dtab + c.p.G + 1; ga.tab_cf = ga.tab_g0 + c.p.G; ga.tab_cl = ga.tab_cf + c.p.NG;
        ga.ssq_in = ssq; ga.n_ssq = h / 32; ga.inv_h = 1.f / h; ga.eps = 1e-5f;
        ga.q_out = out; ga.q_lo_out = out + (32 << 20); ga.kcache = kv; ga.vcache = kv + (size_t)Hkv * S_pad * D * 2; ga.rope_cs = rope;
        ga.Hq = Hq; ga.Hkv = Hkv; ga.L = 512; ga.S_pad = S_pad;
        ga.x_in = x; ga.x = x; ga.xb = out; ga.gain_next = gain; ga.ssq_out = ssq; ga.act = out; ga.logits = (float*)out; ga.Vpad = c.p.n_strips * 32;
        ga.mark = 1; ga.spin_limit = 20000; ga.fault = fault;
        if (woff + c.p.tiled > wbytes) woff = 0;     // rotate: the next launch reads memory no cache holds
        ga.Wt = (const uint4*)(W + woff); woff += rup(c.p.tiled, 4096);
        return ga;
    };
    float ms;
    printf("shape: hidden %d, FFN %d, heads %d/%d x %d, vocabulary %d; %d tokens; %d workgroups of 256 threads\n", h, F, Hq, Hkv, D, V, Tp, nwg);

    {   // launch floor
        GemmArgs ga = args_of(cases[0]);
        for (int rep = 0; rep < 3; ++rep) hipLaunchKernelGGL(k_empty, dim3(256), dim3(256), FV_PAIRED_SMEM_FLOATS(FV_PROBE_TB) * 4, 0, ga);
        CK(hipEventRecord(e0));
        for (int rep = 0; rep < 100; ++rep) hipLaunchKernelGGL(k_empty, dim3(256), dim3(256), FV_PAIRED_SMEM_FLOATS(FV_PROBE_TB) * 4, 0, ga);
        CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1)); CK(hipEventElapsedTime(&ms, e0, e1));
        printf("[floor] empty kernel of the same launch shape, back to back: %.2f us per launch\n", ms * 10);
    }
    for (auto& c : cases) {   // the same bytes as a pure read, one launch per matrix
        for (int rep = 0; rep < 2; ++rep) { GemmArgs g2 = args_of(c); hipLaunchKernelGGL(k_read, dim3(256), dim3(256), 0, 0, g2.Wt, c.p.tiled / 16, (uint4*)out); }
        CK(hipEventRecord(e0));
        for (int rep = 0; rep < 24; ++rep) { GemmArgs g2 = args_of(c); hipLaunchKernelGGL(k_read, dim3(256), dim3(256), 0, 0, g2.Wt, c.p.tiled / 16, (uint4*)out); }
        CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1)); CK(hipEventElapsedTime(&ms, e0, e1));
        printf("[read]  %-8s %6.1f MB  %6.2f us per launch  %5.0f GB/s\n", c.name, c.p.tiled / 1e6, ms * 1e3 / 24, c.p.tiled / (ms / 24) / 1e6);
    }
    for (int g : {32, 64, 128, 192, 256}) {   // what one compute unit can take in: 256 MiB from HBM over fewer workgroups
        const size_t n16 = ((size_t)256 << 20) / 16;
        hipLaunchKernelGGL(k_read, dim3(g), dim3(256), 0, 0, (const uint4*)W, n16, (uint4*)out);
        CK(hipEventRecord(e0));
        for (int rep = 0; rep < 4; ++rep) hipLaunchKernelGGL(k_read, dim3(g), dim3(256), 0, 0, (const uint4*)W + (size_t)(rep + 1) * n16, n16, (uint4*)out);
        CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1)); CK(hipEventElapsedTime(&ms, e0, e1));
        printf("[cu]    256 MiB from HBM over %3d workgroups: %7.1f us  %5.0f GB/s  %5.1f GB/s per compute unit\n", g, ms * 250, 268.4e6 * 4 / ms / 1e6, 268.4e6 * 4 / ms / 1e6 / g);
    }
    {   // the same from L2: every workgroup reads one 512 KiB region 64 times
        const size_t n16 = ((size_t)512 << 10) / 16;
        hipLaunchKernelGGL(k_reread, dim3(256), dim3(256), 0, 0, (const uint4*)X, n16, 4, (uint4*)out);
        CK(hipEventRecord(e0));
        hipLaunchKernelGGL(k_reread, dim3(256), dim3(256), 0, 0, (const uint4*)X, n16, 64, (uint4*)out);
        CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1)); CK(hipEventElapsedTime(&ms, e0, e1));
        printf("[cu]    512 KiB re-read 64 times by each of 256 workgroups (L2 hits): %7.1f us  %5.1f GB/s per compute unit\n", ms * 1e3, 524288.0 * 64 / ms / 1e6);
    }
    for (auto& c : cases) {   // the GEMM, one matrix at a time, 24 launches back to back
        for (int rep = 0; rep < 3; ++rep) launch_epi(c.epi, args_of(c));
        CK(hipEventRecord(e0));
        for (int rep = 0; rep < 24; ++rep) launch_epi(c.epi, args_of(c));
        CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1)); CK(hipEventElapsedTime(&ms, e0, e1));
        printf("[gemm]  %-8s %6.1f MB  %6.2f us per launch  %5.0f GB/s   (%d row groups x %d stages over %d workgroups: %.2f groups each%s)\n", c.name,
               c.bytes / 1e6, ms * 1e3 / 24, c.bytes / (ms / 24) / 1e6, c.p.NG, c.p.NB, c.p.G, (double)c.p.NG / c.p.G, c.p.aligned ? ", whole groups" : "");
#ifdef FV_PROBE_STAMPS
        CK(hipMemset(dts, 0, 1024 * 16 * 8));
        launch_epi(c.epi, args_of(c)); CK(hipDeviceSynchronize());
        std::vector<long long> ts(1024 * 16); CK(hipMemcpy(ts.data(), dts, ts.size() * 8, hipMemcpyDeviceToHost));
        long long t0 = 1LL << 62;
        for (int w = 0; w < c.p.G * 4; ++w) if (ts[w * 16] && ts[w * 16] < t0) t0 = ts[w * 16];
        const char* nm[8] = {"kernel entry", "statistics loads issued", "split computed, request stream positioned", "first stage requested",
                             "three stages requested", "RMSNorm factors reduced, streaming loop entered", "first segment streamed, sums in LDS",
                             "last segment finished (exchange, epilogue)"};
        // wall_clock64 counts at 100 MHz
        for (int k = 0; k < 8; ++k) {
            double mn = 1e18, mx = -1e18, av = 0; int n = 0;
            for (int w = 0; w < c.p.G * 4; ++w) {
                if (!ts[w * 16 + k]) continue;
                const double v = (ts[w * 16 + k] - t0) / 100.0;
                mn = v < mn ? v : mn; mx = v > mx ? v : mx; av += v; ++n;
            }
            if (n) printf("          stamp %d  %-50s  wavefronts %4d   min %6.2f  mean %6.2f  max %6.2f us\n", k, nm[k], n, mn, av / n, mx);
        }
#endif
    }
    {   // the same launches on weights that a pure read has just pulled through the memory-side cache
        for (int ci : {0, 2, 3}) {
            Case& c = cases[ci];
            for (int warm = 0; warm < 2; ++warm) {
                float tot = 0;
                for (int rep = 0; rep < 12; ++rep) {
                    GemmArgs ga = args_of(c);
                    if (warm) hipLaunchKernelGGL(k_read, dim3(256), dim3(256), 0, 0, ga.Wt, c.p.tiled / 16, (uint4*)out);
                    CK(hipEventRecord(e0)); launch_epi(c.epi, ga); CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
                    CK(hipEventElapsedTime(&ms, e0, e1));
                    if (rep >= 2) tot += ms;
                }
                printf("[cache] %-8s %s: %6.2f us (single launches between events)\n", c.name, warm ? "weights just read " : "weights from HBM  ", tot * 100);
            }
        }
    }
    for (int rep = 0; rep < 2; ++rep) {   // a layer's four GEMMs in sequence, 32 layers
        CK(hipEventRecord(e0));
        for (int l = 0; l < 32; ++l) for (int i = 0; i < 4; ++i) launch_epi(cases[i].epi, args_of(cases[i]));
        CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1)); CK(hipEventElapsedTime(&ms, e0, e1));
        const double lb = (double)(cases[0].bytes + cases[1].bytes + cases[2].bytes + cases[3].bytes);
        printf("[layer] 32 x (QKV, O, gate/up, down): %.3f ms  %.1f us per layer  %.0f GB/s\n", ms, ms * 1e3 / 32, lb * 32 / ms / 1e6);
    }
    {   // the same 128 launches as one captured graph, replayed (does the launch path between kernels cost anything?)
        hipStream_t cs; CK(hipStreamCreate(&cs));
        g_stream = cs;
        hipGraph_t graph; hipGraphExec_t exec;
        CK(hipStreamBeginCapture(cs, hipStreamCaptureModeGlobal));
        for (int l = 0; l < 32; ++l) for (int i = 0; i < 4; ++i) launch_epi(cases[i].epi, args_of(cases[i]));
        CK(hipStreamEndCapture(cs, &graph));
        CK(hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0));
        for (int rep = 0; rep < 3; ++rep) {
            CK(hipEventRecord(e0, cs));
            for (int l = 0; l < 32; ++l) for (int i = 0; i < 4; ++i) launch_epi(cases[i].epi, args_of(cases[i]));
            CK(hipEventRecord(e1, cs)); CK(hipEventSynchronize(e1)); CK(hipEventElapsedTime(&ms, e0, e1));
            printf("[graph] 128 launches on a stream : %.3f ms  %.1f us per layer\n", ms, ms * 1e3 / 32);
            CK(hipEventRecord(e0, cs));
            CK(hipGraphLaunch(exec, cs));
            CK(hipEventRecord(e1, cs)); CK(hipEventSynchronize(e1)); CK(hipEventElapsedTime(&ms, e0, e1));
            printf("[graph] the same as a graph      : %.3f ms  %.1f us per layer\n", ms, ms * 1e3 / 32);
        }
        g_stream = nullptr;
        CK(hipGraphExecDestroy(exec)); CK(hipGraphDestroy(graph)); CK(hipStreamDestroy(cs));
    }
    unsigned hf = 0; CK(hipMemcpy(&hf, fault, 4, hipMemcpyDeviceToHost));
    if (hf) printf("a partial tile did not arrive in time\n");
    return hf ? 1 : 0;
}
