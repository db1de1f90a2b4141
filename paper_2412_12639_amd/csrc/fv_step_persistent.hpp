// All decoder layers of one verification step in ONE persistent kernel (up to 64 tokens).
//
// One workgroup per compute unit, launched cooperatively (the runtime refuses the launch unless
// every workgroup is resident), loops over the layers; the phases of a layer -- QKV GEMM, tree
// attention, O GEMM, gate/up GEMM, down GEMM -- are separated by a grid barrier instead of a
// kernel boundary, which costs about a third of one.
//
// Visibility across workgroups inside a launch.  The XCDs' L2 caches are not coherent with each
// other, and a whole-L2 write-back / invalidate per workgroup per phase is far too slow.  So
//   * every buffer that one phase writes and a later phase reads has its OWN address range per
//     layer (the buffers rotate), so no reader can hold a stale line of it from earlier in the
//     launch, and plain cached loads are safe;
//   * producers write such buffers with agent-scope atomic stores (write-through) and wait for
//     them to be acknowledged before they arrive at the barrier;
//   * barrier flags, tickets and partial tiles are read with agent-scope atomic loads.
#pragma once
// (included from fv_kernels.hpp after the GEMM and attention bodies)

struct PersistGemm {          // stream-K plan of one GEMM type
    int NG, NB, G, segmax, n_strips, aligned;
    const int* tab;           // u0[G+1], g0[G], cf[NG], cl[NG]
};

struct PersistArgs {
    int n_layers, T, Tp, L, h, Hq, Hkv, S_pad, n_ssq;
    float inv_h, eps, scale;
    const char* w_layers;     // tiled weights of layer 0; layer stride and per-matrix offsets follow
    size_t layer_w_bytes, off_w[4];
    char* kc; char* vc; size_t kv_layer_bytes;
    const float* gains;       // [2*NL+1][h]: attn gain, mlp gain per layer, then the final gain
    const float2* rope_cs;
    const uint64_t* mask;
    // rotating activations: one slot per layer (+1), offsets of each buffer inside a slot
    char* rot; size_t rot_stride, o_xa, o_xm, o_xba, o_xbm, o_ssqa, o_ssqm, o_q, o_attn, o_act;
    float* part; unsigned part_bytes; int* tickets; const uint4* zeros;
    float* attn_part; int* attn_tickets; int attn_ks;
    unsigned* bar;            // [0] release word, slots at bar[64 + 32*b]
    unsigned gen0;            // barrier generation before this launch
    int* err;                 // set to 1 if a barrier wait gave up
    long long* tstamp;        // optional [256][16] phase time stamps of layer 1 (100 MHz counter), or null;
                              // a second [256][16] block holds stamps from inside GEMM phase ts_phase
    int ts_phase;
    PersistGemm g[4];         // QKV, O, GU, DN
};

#define FV_SPIN_LIMIT 200000   // polls before a barrier wait gives up (each poll is ~1 us round trip)

// Flag barrier: every workgroup publishes its generation in its own slot; workgroup 0 polls all
// slots in parallel (one thread per slot) and then publishes the release word, which the others
// poll.  Every wait is bounded; a wait that gives up raises *err and the kernel winds down.
__device__ __forceinline__ bool grid_barrier(const PersistArgs& a, unsigned gen, bool& failed) {
    __shared__ int ok_lds;
    const int tid = threadIdx.x;
    const unsigned nblk = gridDim.x;
    unsigned* go = a.bar;
    unsigned* slots = a.bar + 64;
    if (tid == 0) ok_lds = 1;
    __syncthreads();   // every wavefront has waited for its own stores before calling (see callers)
    if (blockIdx.x == 0) {
        // once a wait has given up, workgroup 0 stops waiting for good and only keeps releasing the
        // others, so a lost workgroup costs one bounded wait, not one per barrier
        if (!failed && tid > 0 && (unsigned)tid < nblk) {
            int spins = 0;
            while ((int)(__hip_atomic_load(slots + tid * 32, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - gen) < 0) {
                if (++spins > FV_SPIN_LIMIT) { ok_lds = 0; break; }
                __builtin_amdgcn_s_sleep(2);
            }
        }
        __syncthreads();
        if (!ok_lds) failed = true;
        if (tid == 0) {
            if (!ok_lds) __hip_atomic_store(a.err, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(go, gen, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        __syncthreads();
        return true;   // workgroup 0 always runs to the end (its results are discarded by the host on error)
    }
    if (tid == 0) {
        __hip_atomic_store(slots + blockIdx.x * 32, gen, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        int spins = 0;
        while ((int)(__hip_atomic_load(go, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - gen) < 0) {
            if (++spins > FV_SPIN_LIMIT) { ok_lds = 0; break; }
            __builtin_amdgcn_s_sleep(4);
        }
        if (!ok_lds) __hip_atomic_store(a.err, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    return ok_lds != 0;   // false: the release never came; this workgroup leaves the kernel
}

#define FV_PERSIST_SMEM_FLOATS(TB, D) \
    (FV_PAIRED_SMEM_FLOATS(TB) > FV_ATTN_SMEM_FLOATS(D) ? FV_PAIRED_SMEM_FLOATS(TB) : FV_ATTN_SMEM_FLOATS(D))

// RS: strips per wavefront in the GEMM phases (1: direct form, 2: paired form; the host passes the
// matching split plans).
template <typename EL, int TB, int D, int RS>
__global__ __launch_bounds__(256, 1) void k_step_persistent(PersistArgs a) {
    extern __shared__ __attribute__((aligned(16))) float smem[];   // FV_PERSIST_SMEM_FLOATS(TB, D) floats
    const int wg = blockIdx.x;
    unsigned gen = a.gen0;
    bool failed = false;
    int stamp_i = 0;

    // Arguments of GEMM phase (layer l, k in {0: QKV, 2: O, 3: gate/up, 4: down})
    auto gemm_args = [&](int l, int k) {
        char* rs = a.rot + (size_t)l * a.rot_stride;      // this layer's slot of the rotating buffers
        char* rn = rs + a.rot_stride;                     // next layer's slot
        const int which = (k == 0) ? 0 : k - 1;           // QKV, O, GU, DN
        const PersistGemm& p = a.g[which];
        GemmArgs ga;
        ga.Wt = (const uint4*)(a.w_layers + (size_t)l * a.layer_w_bytes + a.off_w[which]);
        ga.part = a.part; ga.part_bytes = a.part_bytes; ga.tickets = a.tickets; ga.zeros = a.zeros;
        ga.NG = p.NG; ga.NB = p.NB; ga.G = p.G; ga.segmax = p.segmax;
        ga.tab_u0 = p.tab; ga.tab_g0 = p.tab + p.G + 1; ga.tab_cf = ga.tab_g0 + p.G; ga.tab_cl = ga.tab_cf + p.NG;
        ga.T = a.T; ga.n_strips = p.n_strips;
        ga.n_ssq = a.n_ssq; ga.inv_h = a.inv_h; ga.eps = a.eps;
        ga.Hq = a.Hq; ga.Hkv = a.Hkv; ga.L = a.L; ga.S_pad = a.S_pad; ga.rope_cs = a.rope_cs;
        ga.kcache = a.kc + (size_t)l * a.kv_layer_bytes; ga.vcache = a.vc + (size_t)l * a.kv_layer_bytes;
        ga.q_out = rs + a.o_q; ga.act = rs + a.o_act;
        ga.logits = nullptr; ga.Vpad = 0; ga.aligned = p.aligned;
        ga.x_in = nullptr; ga.x = nullptr; ga.xb = nullptr; ga.gain_next = nullptr; ga.ssq_out = nullptr; ga.ssq_in = nullptr;
        if (k == 0) {          // normalised input of the layer -> rotated q, k/v into the cache
            ga.epi = EPI_QKV;
            ga.X = (const uint4*)(rs + a.o_xba); ga.ssq_in = (const float*)(rs + a.o_ssqa);
        } else if (k == 2) {   // output projection + residual, input and statistics of the FFN norm
            ga.epi = EPI_RESID;
            ga.X = (const uint4*)(rs + a.o_attn);
            ga.x_in = (const float*)(rs + a.o_xa); ga.x = (float*)(rs + a.o_xm);
            ga.xb = rs + a.o_xbm; ga.gain_next = a.gains + (size_t)(2 * l + 1) * a.h; ga.ssq_out = (float*)(rs + a.o_ssqm);
        } else if (k == 3) {   // gate / up + SwiGLU
            ga.epi = EPI_SWIGLU;
            ga.X = (const uint4*)(rs + a.o_xbm); ga.ssq_in = (const float*)(rs + a.o_ssqm);
        } else {               // down projection + residual -> next layer's (or the head's) input
            ga.epi = EPI_RESID;
            ga.X = (const uint4*)(rs + a.o_act);
            ga.x_in = (const float*)(rs + a.o_xm); ga.x = (float*)(rn + a.o_xa);
            ga.xb = rn + a.o_xba; ga.gain_next = a.gains + (size_t)(2 * l + 2) * a.h; ga.ssq_out = (float*)(rn + a.o_ssqa);
        }
        return ga;
    };

    // Phases 0..4 of layer l: QKV, attention, O, gate/up, down.  One loop, so that the GEMM body
    // (the bulk of the code) is instantiated once and the kernel stays inside the instruction cache.
    // The weight tiles of a GEMM phase's first three stages are requested BEFORE the barrier that ends
    // the previous phase (weights do not depend on activations), so HBM works through the barrier.
    // Not across the attention phase, which needs the registers.
    uint4 w[3][FV_FRAGS];
    bool preloaded = false;
    const int n_phases = 5 * a.n_layers;
    for (int ph = 0; ph < n_phases; ++ph) {
        const int l = ph / 5, k = ph - 5 * l;
        if (k == 1) {
            // tree attention: (head, 32-node block, key part) units round-robin over the workgroups.
            // (Nothing is prefetched across this phase: say so, or the weight registers stay reserved.)
#pragma unroll
            for (int i = 0; i < 3; ++i)
#pragma unroll
                for (int f = 0; f < FV_FRAGS; ++f) w[i][f] = make_uint4(0u, 0u, 0u, 0u);
            char* rs = a.rot + (size_t)l * a.rot_stride;
            AttnArgs aa;
            aa.q = (const uint4*)(rs + a.o_q);
            aa.kc = (const uint4*)(a.kc + (size_t)l * a.kv_layer_bytes);
            aa.vc = (const uint4*)(a.vc + (size_t)l * a.kv_layer_bytes);
            aa.out = rs + a.o_attn; aa.mask = a.mask;
            aa.Tp = a.Tp; aa.T = a.T; aa.L = a.L; aa.Hq = a.Hq; aa.Hkv = a.Hkv; aa.S_pad = a.S_pad; aa.scale = a.scale;
            aa.ks = a.attn_ks; aa.part = a.attn_part; aa.tickets = a.attn_tickets;
            const int units = a.Hq * TB * a.attn_ks;
            for (int it = wg; it < units; it += gridDim.x) {
                attn_body<EL, D, true>(aa, it / a.attn_ks, it % a.attn_ks, smem);
                __syncthreads();
            }
        } else {
            GemmArgs ga = gemm_args(l, k);
            gemm_direct_body<EL, TB, D, -1, true, RS>(ga, wg, smem, w, preloaded);
            preloaded = false;
        }
        if (ph + 1 < n_phases) {
            __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): this lane's stores are out
            if (k != 0) {   // the next phase is a GEMM
                const int k2 = (k == 4) ? 0 : k + 1, l2 = (k == 4) ? l + 1 : l;
                const GemmArgs gn = gemm_args(l2, k2);
                gemm_direct_prefetch<RS>(gn, wg, w);
                preloaded = true;
            }
            if (a.tstamp && l == 1 && threadIdx.x == 0) a.tstamp[blockIdx.x * 16 + (stamp_i++)] = wall_clock64();
            if (!grid_barrier(a, ++gen, failed)) return;
            if (a.tstamp && l == 1 && threadIdx.x == 0) a.tstamp[blockIdx.x * 16 + (stamp_i++)] = wall_clock64();
        }
    }
}
