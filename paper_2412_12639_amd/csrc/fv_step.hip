// The kernel sequence of one decoder pass and the helpers that launch kernels, for ONE
// (element type, head size) pair: compiled with -DFV_INST_EL=BF16|F32 -DFV_INST_D=64|128.
#include "fv_host.hpp"
#include "fv_kernels.hpp"

#include <algorithm>
#include <cmath>
#include <cstring>

struct PhaseTimer {   // brackets launches with events when profiling is on
    fv_ctx* c; int phase; size_t idx = 0; bool on;
    PhaseTimer(fv_ctx* c_, int ph) : c(c_), phase(ph), on(c_->profiling) {
        if (!on) return;
        if (c->pev_used + 2 > c->pev.size()) {
            for (int i = 0; i < 2; ++i) { hipEvent_t e; if (hipEventCreate(&e) != hipSuccess) { on = false; return; } c->pev.push_back(e); }
            c->pev_phase.push_back(phase);
        }
        idx = c->pev_used;
        c->pev_phase[idx / 2] = phase;
        c->pev_used += 2;
        (void)hipEventRecord(c->pev[idx], c->stream);
    }
    ~PhaseTimer() { if (on) (void)hipEventRecord(c->pev[idx + 1], c->stream); }
};

template <typename EL, int TB, int D, int EPI>
int launch_gemm_t(fv_ctx* c, const GemmArgs& ga0) {
    const size_t lds = (size_t)2 * TB * 32 * 256;
    GemmArgs ga = ga0;
    // At 128 / 256 tokens the projections with heavy fix-ups (QKV: rotary epilogue on 4 / 8 tiles per
    // wavefront; O and down: 8 contributors per row group) leave the reduction to k_gemm_fix.
    ga.defer = (TB >= 4 && ((c->gemm_fix == 1 && (EPI == EPI_QKV || EPI == EPI_RESID)) || c->gemm_fix == 2) && ga.n_fix > 0) ? 1 : 0;
    hipLaunchKernelGGL((k_gemm<EL, TB, D, EPI>), dim3(ga.G), dim3(64 * FV_R), lds, c->stream, ga);
    if (hipGetLastError() != hipSuccess) return FV_E_HIP;
    if (ga.defer) {
        const int tiles = ga.n_fix * FV_R * TB;
        hipLaunchKernelGGL((k_gemm_fix<EL, TB, D, EPI>), dim3((tiles + 3) / 4), dim3(256), 0, c->stream, ga);
        if (hipGetLastError() != hipSuccess) return FV_E_HIP;
    }
    return FV_OK;
}

template <typename EL, int TB, int D, int EPI>
int launch_gemm_direct_t(fv_ctx* c, const GemmArgs& ga) {
    hipLaunchKernelGGL((k_gemm_direct<EL, TB, D, EPI>), dim3(ga.G), dim3(256), FV_DIRECT_SMEM_FLOATS(TB) * 4, c->stream, ga);
    return hipGetLastError() == hipSuccess ? FV_OK : FV_E_HIP;
}

// GEMM kernel used up to 64 tokens (above that always the shared-activation kernel)

template <typename EL, int TB, int D, int EPI>
int launch_gemm_paired_t(fv_ctx* c, const GemmArgs& ga) {
    hipLaunchKernelGGL((k_gemm_paired<EL, TB, D, EPI>), dim3(ga.G), dim3(256), FV_PAIRED_SMEM_FLOATS(TB) * 4, c->stream, ga);
    return hipGetLastError() == hipSuccess ? FV_OK : FV_E_HIP;
}

// The direct and paired kernels need the partial area all zeros when they start and leave it so; the
// shared-activation kernel (and a step that ran into the time-out) leaves partial sums behind.  `scr` is the
// scratch `ga.part` belongs to: its host flag says which of the two states the area is in.
template <typename EL, int D, int EPI>
int launch_gemm(fv_ctx* c, int Tp, const GemmArgs& ga, int kind, const StepScratch* scr) {
    const bool marked = (kind == GEMM_DIRECT || kind == GEMM_PAIRED) && Tp <= 64;
    if (scr && scr->dirty) {
        if (marked && *scr->dirty) {
            const size_t n = scr->part_bytes / 4;
            hipLaunchKernelGGL(k_zero_words<0>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, c->stream, (uint32_t*)scr->part, n);
            if (hipGetLastError() != hipSuccess) return FV_E_HIP;
            *scr->dirty = false;
        }
        if (!marked) *scr->dirty = true;
    }
    if (kind == GEMM_DIRECT) return Tp == 32 ? launch_gemm_direct_t<EL, 1, D, EPI>(c, ga) : launch_gemm_direct_t<EL, 2, D, EPI>(c, ga);
    if (kind == GEMM_PAIRED) return Tp == 32 ? launch_gemm_paired_t<EL, 1, D, EPI>(c, ga) : launch_gemm_paired_t<EL, 2, D, EPI>(c, ga);
    switch (Tp) {
        case 32: return launch_gemm_t<EL, 1, D, EPI>(c, ga);
        case 64: return launch_gemm_t<EL, 2, D, EPI>(c, ga);
        case 128: return launch_gemm_t<EL, 4, D, EPI>(c, ga);
        case 256: return launch_gemm_t<EL, 8, D, EPI>(c, ga);
    }
    return FV_E_BAD_ARG;
}

template <typename EL, int D, int EPI>
int set_gemm_attrs_e() {
    // the 256-token instantiation double-buffers 2 x 64 KiB of activations in LDS
    HIPCHK(hipFuncSetAttribute((const void*)k_gemm<EL, 8, D, EPI>, hipFuncAttributeMaxDynamicSharedMemorySize, 2 * 256 * 256));
    HIPCHK(hipFuncSetAttribute((const void*)k_gemm<EL, 4, D, EPI>, hipFuncAttributeMaxDynamicSharedMemorySize, 2 * 128 * 256));
    HIPCHK(hipFuncSetAttribute((const void*)k_gemm_direct<EL, 1, D, EPI>, hipFuncAttributeMaxDynamicSharedMemorySize, FV_DIRECT_SMEM_FLOATS(1) * 4));
    HIPCHK(hipFuncSetAttribute((const void*)k_gemm_direct<EL, 2, D, EPI>, hipFuncAttributeMaxDynamicSharedMemorySize, FV_DIRECT_SMEM_FLOATS(2) * 4));
    HIPCHK(hipFuncSetAttribute((const void*)k_gemm_paired<EL, 1, D, EPI>, hipFuncAttributeMaxDynamicSharedMemorySize, FV_PAIRED_SMEM_FLOATS(1) * 4));
    HIPCHK(hipFuncSetAttribute((const void*)k_gemm_paired<EL, 2, D, EPI>, hipFuncAttributeMaxDynamicSharedMemorySize, FV_PAIRED_SMEM_FLOATS(2) * 4));
    return FV_OK;
}
template <typename EL, int D>
int set_gemm_attrs_d() {
    HIPCHK(hipFuncSetAttribute((const void*)k_attn_canon<EL, D>, hipFuncAttributeMaxDynamicSharedMemorySize,
                               FV_CANON_SMEM_BYTES(D, Tr<EL>::ESZ)));
    int rc = set_gemm_attrs_e<EL, D, EPI_QKV>();
    if (!rc) rc = set_gemm_attrs_e<EL, D, EPI_RESID>();
    if (!rc) rc = set_gemm_attrs_e<EL, D, EPI_SWIGLU>();
    if (!rc) rc = set_gemm_attrs_e<EL, D, EPI_LOGITS>();
    return rc;
}
// Key split of the attention: enough workgroups per (head, node block) item to cover the CUs,
// but at least two 32-key blocks each.
static int attn_key_split(int items, int n_keys, int n_wg) {
    int ks = n_wg / (items > 0 ? items : 1);
    const int nkb = (n_keys + 31) / 32;
    if (ks > nkb / 2) ks = nkb / 2;
    if (ks > 8) ks = 8;
    if (ks < 1) ks = 1;
    return ks;
}

// Step-independent attention (fv_attn_canon.hpp): taken by verification steps (one-token steps are
// verification steps of a one-node tree) of up to 64 rows whose nodes are at most FV_CANON_DEPTH
// deep, when the far parts fit the triple slots of the scratch in use.  Fills everything of `ca`
// that does not change from layer to layer and returns true, or returns false (k_attn then).
template <typename EL, int D>
static bool plan_canon_attention(const fv_ctx* c, int T, int Tp, StepMode mode, CanonArgs& ca) {
    if (!c->attn_canon || (mode != STEP_VERIFY && mode != STEP_VERIFY_SAMPLED) || Tp > 64) return false;
    int maxdepth = 0;
    for (int i = 0; i < T; ++i) maxdepth = std::max(maxdepth, (int)c->h_in[2 * FV_MAX_TREE + i]);
    if (maxdepth > FV_CANON_DEPTH) return false;
    const fv_cfg& cf = c->cfg;
    const int L = c->cur_len;
    const int pb = (L + maxdepth) >> 5;
    const int nfb = pb > 0 ? pb - 1 : 0, np = canon_parts(nfb);
    if (np > FV_CANON_MAX_PARTS || np + 1 > c->scr->aslots) return false;
    memset(&ca, 0, sizeof(ca));
    ca.Tp = Tp; ca.T = T; ca.L = L; ca.Hq = cf.n_q_heads; ca.Hkv = cf.n_kv_heads; ca.S_pad = c->lay.S_pad;
    ca.scale = 1.f / std::sqrt((float)D);
    ca.nfb = nfb; ca.np = np;
    const int items = cf.n_q_heads * (Tp / 32);
    int kw = 256 / items;
    ca.kw = kw < 1 ? 1 : kw > 8 ? 8 : kw;
    // parts to workgroups: heaviest first, each to the least loaded workgroup
    int load[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int j = np - 1; j >= 0; --j) {
        int best = 0;
        for (int w = 1; w < ca.kw; ++w) if (load[w] < load[best]) best = w;
        ca.owner[j] = (unsigned char)best;
        load[best] += canon_part_run(j) + 1;   // a run of blocks plus the part's merge
    }
    ca.pos = c->at<int32_t>(c->lay.off_pos); ca.anc = c->at<uint8_t>(c->lay.off_anc);
    ca.part = c->scr->apart; ca.tickets = c->scr->atick;
    return true;
}

// One pass of the decoder over T new rows whose tokens/parent/depth are in c->h_in.
template <typename EL, int D>
int run_step(fv_ctx* c, int T, StepMode mode) {
    const fv_cfg& cf = c->cfg;
    const Layout& ly = c->lay;
    const int Tp = pad_tokens(T);
    const int L = c->cur_len;
    const int h = cf.hidden;
    hipStream_t st = c->stream;
    c->pev_used = 0;

    HIPCHK(hipMemcpyAsync(c->at<int32_t>(ly.off_stepin), c->h_in, 3 * FV_MAX_TREE * 4, hipMemcpyHostToDevice, st));
    if (mode == STEP_VERIFY_SAMPLED)
        HIPCHK(hipMemcpyAsync(c->at<double>(ly.off_unif), c->h_unif, 2 * FV_MAX_TREE * 8, hipMemcpyHostToDevice, st));
    HIPCHK(hipEventRecord(c->ev0, st));
    {
        PhaseTimer pt(c, FV_PH_OTHER);
        IngestArgs ia;
        ia.tok_in = c->at<int32_t>(ly.off_stepin); ia.cap = FV_MAX_TREE; ia.T = T; ia.Tp = Tp; ia.L = L; ia.half_d = D / 2;
        ia.log2_base = std::log2((double)cf.rope_base);
        ia.mask = c->at<uint64_t>(ly.off_mask); ia.pos = c->at<int32_t>(ly.off_pos); ia.rope_cs = c->at<float2>(ly.off_rope);
        ia.anc = c->at<uint8_t>(ly.off_anc);
        hipLaunchKernelGGL(k_ingest, dim3((Tp + 3) / 4), dim3(256), 0, st, ia);
        EmbedArgs ea;
        ea.table = c->at<void>(ly.off_embed); ea.tok = c->at<int32_t>(ly.off_stepin); ea.gain = c->gain(0);
        ea.x = c->at<float>(ly.off_x);
        ea.xb = c->at<void>(ly.off_xb);
        ea.ssq_part = c->at<float>(ly.off_ssq);
        ea.h = h; ea.T = T; ea.Tp = Tp;
        hipLaunchKernelGGL((k_embed<EL>), dim3(h / 32), dim3(Tp < 64 ? 64 : Tp), 0, st, ea);
    }
    HIPCHK(hipGetLastError());

    // kernel per matrix: above 64 tokens always the shared-activation kernel
    auto kind_of = [&](int which) { return (Tp <= 64) ? c->kind[which] : (int)GEMM_SHARED; };
    auto gemm_args = [&](int which, const void* Wt, size_t x_off) {
        const int kind = kind_of(which);
        const GemmPlan& p = (kind == GEMM_DIRECT) ? ly.gd[which] : (kind == GEMM_PAIRED) ? ly.gp[which] : ly.gm[which];
        GemmArgs ga;
        memset(&ga, 0, sizeof(ga));
        ga.Wt = (const uint4*)Wt; ga.X = c->at<uint4>(x_off); ga.part = c->scr->part; ga.part_bytes = c->scr->part_bytes;
        ga.tickets = c->scr->tickets; ga.zeros = c->at<uint4>(ly.off_zeros);
        ga.NG = p.NG; ga.NB = p.NB; ga.G = p.G; ga.segmax = p.segmax; ga.aligned = p.aligned;
        ga.tab_u0 = c->at<int>(p.off_tab); ga.tab_g0 = ga.tab_u0 + p.G + 1; ga.tab_cf = ga.tab_g0 + p.G; ga.tab_cl = ga.tab_cf + p.NG;
        ga.fix_groups = (const int4*)(ga.tab_u0 + (((size_t)2 * p.G + 1 + 2 * p.NG + 3) & ~(size_t)3)); ga.n_fix = p.n_fix; ga.rinv_out = c->at<float>(ly.off_rinv);
        ga.T = T; ga.n_strips = p.n_strips;
        ga.ssq_in = c->at<float>(ly.off_ssq); ga.n_ssq = h / 32; ga.inv_h = 1.f / (float)h; ga.eps = cf.rms_eps;
        ga.mark = c->exchange_test ? 0u : 1u;   // the test of the time-out leaves the partial tiles unmarked
        ga.spin_limit = c->exchange_test ? 2u : FV_EXCHANGE_SPINS;
        ga.fault = &c->at<FvResult>(ly.off_res)->fault;
        return ga;
    };

    CanonArgs ca;
    const bool canon = plan_canon_attention<EL, D>(c, T, Tp, mode, ca);

    for (int l = 0; l < cf.n_layers; ++l) {
        int rc;
        {   // q, k, v projections of the normalised input, rotary at pos = L + depth, K/V to cache slots L + i
            PhaseTimer pt(c, FV_PH_GEMM);
            GemmArgs ga = gemm_args(GM_QKV, c->layer_w(l, 0), ly.off_xb);
            ga.q_out = c->at<void>(ly.off_q); ga.q_lo_out = c->at<void>(ly.off_qlo); ga.kcache = c->kc(l); ga.vcache = c->vc(l);
            ga.rope_cs = c->at<float2>(ly.off_rope); ga.Hq = cf.n_q_heads; ga.Hkv = cf.n_kv_heads; ga.L = L; ga.S_pad = ly.S_pad;
            rc = launch_gemm<EL, D, EPI_QKV>(c, Tp, ga, kind_of(GM_QKV), c->scr);
            if (rc) return rc;
        }
        if (canon) {
            PhaseTimer pt(c, FV_PH_ATTN);
            ca.q = c->at<uint4>(ly.off_q); ca.q_lo = c->at<uint4>(ly.off_qlo); ca.kc = (const uint4*)c->kc(l); ca.vc = (const uint4*)c->vc(l);
            ca.out = c->at<void>(ly.off_attn);
            hipLaunchKernelGGL((k_attn_canon<EL, D>), dim3(cf.n_q_heads * (Tp / 32) * ca.kw), dim3(256),
                               FV_CANON_SMEM_BYTES(D, Tr<EL>::ESZ), st, ca);
            HIPCHK(hipGetLastError());
        } else {
            PhaseTimer pt(c, FV_PH_ATTN);
            AttnArgs aa;
            aa.q = c->at<uint4>(ly.off_q); aa.q_lo = c->at<uint4>(ly.off_qlo); aa.kc = (const uint4*)c->kc(l); aa.vc = (const uint4*)c->vc(l);
            aa.out = c->at<void>(ly.off_attn); aa.mask = c->at<uint64_t>(ly.off_mask);
            aa.Tp = Tp; aa.T = T; aa.TK = T; aa.L = L; aa.Hq = cf.n_q_heads; aa.Hkv = cf.n_kv_heads; aa.S_pad = ly.S_pad;
            aa.scale = 1.f / std::sqrt((float)D);
            aa.ks = attn_key_split(cf.n_q_heads * (Tp / 32), L + T, 256);
            aa.part = c->scr->apart; aa.tickets = c->scr->atick;
            hipLaunchKernelGGL((k_attn<EL, D>), dim3(cf.n_q_heads * (Tp / 32) * aa.ks), dim3(256), 0, st, aa);
            HIPCHK(hipGetLastError());
        }
        {   // output projection, residual add, statistics + input of the FFN norm
            PhaseTimer pt(c, FV_PH_GEMM);
            GemmArgs ga = gemm_args(GM_O, c->layer_w(l, 1), ly.off_attn);
            ga.x_in = ga.x = c->at<float>(ly.off_x); ga.xb = c->at<void>(ly.off_xb); ga.gain_next = c->gain(2 * l + 1);
            ga.ssq_out = c->at<float>(ly.off_ssq);
            rc = launch_gemm<EL, D, EPI_RESID>(c, Tp, ga, kind_of(GM_O), c->scr);
            if (rc) return rc;
        }
        {   // gate and up projections, SwiGLU
            PhaseTimer pt(c, FV_PH_GEMM);
            GemmArgs ga = gemm_args(GM_GU, c->layer_w(l, 2), ly.off_xb);
            ga.act = c->at<void>(ly.off_act);
            rc = launch_gemm<EL, D, EPI_SWIGLU>(c, Tp, ga, kind_of(GM_GU), c->scr);
            if (rc) return rc;
        }
        {   // down projection, residual add, statistics + input of the next norm
            PhaseTimer pt(c, FV_PH_GEMM);
            GemmArgs ga = gemm_args(GM_DN, c->layer_w(l, 3), ly.off_act);
            ga.x_in = ga.x = c->at<float>(ly.off_x); ga.xb = c->at<void>(ly.off_xb);
            ga.gain_next = (l + 1 < cf.n_layers) ? c->gain(2 * (l + 1)) : c->gain(2 * cf.n_layers);
            ga.ssq_out = c->at<float>(ly.off_ssq);
            rc = launch_gemm<EL, D, EPI_RESID>(c, Tp, ga, kind_of(GM_DN), c->scr);
            if (rc) return rc;
        }
    }

    if (mode != STEP_PREFILL_MID) {
        {
            PhaseTimer pt(c, FV_PH_GEMM);
            GemmArgs ga = gemm_args(GM_LM, c->at<void>(ly.off_lm), ly.off_xb);
            ga.logits = c->at<float>(ly.off_logits); ga.Vpad = ly.Vpad;
            int rc = launch_gemm<EL, D, EPI_LOGITS>(c, Tp, ga, kind_of(GM_LM), c->scr);
            if (rc) return rc;
        }
        PhaseTimer pt(c, FV_PH_OTHER);
        ArgmaxArgs am;
        am.logits = c->at<float>(ly.off_logits); am.am = c->at<int32_t>(ly.off_am); am.V = cf.vocab; am.Vpad = ly.Vpad;
        hipLaunchKernelGGL(k_argmax, dim3(T), dim3(256), 0, st, am);
        if (mode == STEP_VERIFY_SAMPLED) {
            SampledArgs sa;
            sa.tok_in = c->at<int32_t>(ly.off_stepin); sa.cap = FV_MAX_TREE; sa.T = T;
            sa.logits = c->at<float>(ly.off_logits); sa.V = cf.vocab; sa.Vpad = ly.Vpad;
            sa.inv_temperature = c->sample_inv_temperature; sa.draft_probs = c->sample_draft;
            sa.u_accept = c->at<double>(ly.off_unif); sa.u_sample = sa.u_accept + FV_MAX_TREE;
            sa.work = c->at<double>(ly.off_pwork); sa.res = c->at<FvResult>(ly.off_res);
            hipLaunchKernelGGL(k_accept_sampled, dim3(1), dim3(FV_SAMPLED_THREADS), 0, st, sa);
        }
        if (mode == STEP_VERIFY) {
            ScanArgs sa;
            sa.tok_in = c->at<int32_t>(ly.off_stepin); sa.cap = FV_MAX_TREE; sa.T = T;
            sa.mask = c->at<uint64_t>(ly.off_mask); sa.am = c->at<int32_t>(ly.off_am); sa.res = c->at<FvResult>(ly.off_res);
            hipLaunchKernelGGL(k_scan, dim3(1), dim3(256), 0, st, sa);
        }
        if (mode == STEP_VERIFY || mode == STEP_VERIFY_SAMPLED) {
            CompactArgs ca;
            ca.kcache = c->at<void>(ly.off_k); ca.vcache = c->at<void>(ly.off_v); ca.res = c->at<FvResult>(ly.off_res);
            ca.L = L; ca.S_pad = ly.S_pad;
            hipLaunchKernelGGL((k_compact<EL, D>), dim3(cf.n_layers * cf.n_kv_heads), dim3(D), 0, st, ca);
            // features of the accepted path (what the drafter is given next to the tokens)
            FeatureArgs fa;
            fa.res = c->at<FvResult>(ly.off_res);
            fa.x = c->at<float>(ly.off_x);
            fa.ssq = c->at<float>(ly.off_ssq);
            fa.gain = c->gain(2 * cf.n_layers); fa.out = c->at<float>(ly.off_feat);
            fa.h = h; fa.Tp = Tp; fa.inv_h = 1.f / (float)h; fa.eps = cf.rms_eps;
            hipLaunchKernelGGL(k_features, dim3(T), dim3(256), 0, st, fa);
        }
        HIPCHK(hipGetLastError());
    }
    HIPCHK(hipEventRecord(c->ev1, st));
    if (mode == STEP_VERIFY || mode == STEP_VERIFY_SAMPLED)
        HIPCHK(hipMemcpyAsync(c->h_res, c->at<FvResult>(ly.off_res), sizeof(FvResult), hipMemcpyDeviceToHost, st));
    else {
        if (mode == STEP_PREFILL_LAST)
            HIPCHK(hipMemcpyAsync(&c->h_res->next_token, c->at<int32_t>(ly.off_am) + (T - 1), 4, hipMemcpyDeviceToHost, st));
        HIPCHK(hipMemcpyAsync(&c->h_res->fault, &c->at<FvResult>(ly.off_res)->fault, 4, hipMemcpyDeviceToHost, st));
    }
    HIPCHK(hipStreamSynchronize(st));
    if (c->h_res->fault) {
        if (c->scr->dirty) *c->scr->dirty = true;   // unconsumed partial tiles may be left behind
        return FV_E_EXCHANGE_TIMEOUT;
    }
    HIPCHK(hipEventElapsedTime(&c->last_ms, c->ev0, c->ev1));
    if (c->profiling) {
        for (size_t i = 0; i + 1 < c->pev_used; i += 2) {
            float ms = 0.f;
            if (hipEventElapsedTime(&ms, c->pev[i], c->pev[i + 1]) == hipSuccess) {
                c->ph_ms[c->pev_phase[i / 2]] += ms;
                c->ph_n[c->pev_phase[i / 2]] += 1;
            }
        }
    }
    c->last_T = T; c->last_Tp = Tp; c->last_L = L;
    c->last_was_verify = (mode == STEP_VERIFY || mode == STEP_VERIFY_SAMPLED);
    return FV_OK;
}

template <typename EL>
int tile_upload(fv_ctx* c, int kind, const GemmPlan& p, char* out, const void* h0, size_t n0, const void* h1, size_t n1,
                const void* h2, size_t n2, int N) {
    const fv_cfg& cf = c->cfg;
    const size_t esz = Tr<EL>::ESZ;
    char* stage = c->arena + c->lay.off_stage;
    if ((n0 + n1 + n2) * esz > c->lay.stage_bytes) return FV_E_BAD_ARG;
    HIPCHK(hipMemcpyAsync(stage, h0, n0 * esz, hipMemcpyHostToDevice, c->stream));
    if (h1) HIPCHK(hipMemcpyAsync(stage + n0 * esz, h1, n1 * esz, hipMemcpyHostToDevice, c->stream));
    if (h2) HIPCHK(hipMemcpyAsync(stage + (n0 + n1) * esz, h2, n2 * esz, hipMemcpyHostToDevice, c->stream));
    TileArgs ta;
    ta.src0 = stage; ta.src1 = stage + n0 * esz; ta.src2 = stage + (n0 + n1) * esz;
    ta.out = (uint4*)out; ta.kind = kind; ta.n_strips_pad = p.n_strips_pad; ta.NB = p.NB; ta.K = p.K; ta.N = N;
    ta.Hq = cf.n_q_heads; ta.Hkv = cf.n_kv_heads; ta.D = cf.head_dim; ta.F = cf.ffn;
    const size_t total = (size_t)p.n_strips_pad * p.NB * FV_FRAGS * 64;
    hipLaunchKernelGGL((k_tile<EL>), dim3((unsigned)((total + 255) / 256)), dim3(256), 0, c->stream, ta);
    HIPCHK(hipGetLastError());
    HIPCHK(hipStreamSynchronize(c->stream));   // the staging area is reused by the next tensor
    return FV_OK;
}

template <typename EL, int D>
int read_kv_t(fv_ctx* c, int layer, int slot0, int n, float* k_out, float* v_out) {
    const fv_cfg& cf = c->cfg;
    const size_t row = (size_t)cf.n_kv_heads * D;
    float* dk = c->at<float>(c->lay.off_kvread);
    float* dv = dk + 64 * row;
    for (int s = 0; s < n; s += 64) {
        const int m = (n - s < 64) ? n - s : 64;
        ReadKvArgs ra;
        ra.kcache = c->kc(layer); ra.vcache = c->vc(layer); ra.k_out = dk; ra.v_out = dv;
        ra.slot0 = slot0 + s; ra.n = m; ra.Hkv = cf.n_kv_heads; ra.S_pad = c->lay.S_pad;
        hipLaunchKernelGGL((k_read_kv<EL, D>), dim3(m, cf.n_kv_heads), dim3(D), 0, c->stream, ra);
        HIPCHK(hipGetLastError());
        HIPCHK(hipMemcpyAsync(k_out + (size_t)s * row, dk, (size_t)m * row * 4, hipMemcpyDeviceToHost, c->stream));
        HIPCHK(hipMemcpyAsync(v_out + (size_t)s * row, dv, (size_t)m * row * 4, hipMemcpyDeviceToHost, c->stream));
        HIPCHK(hipStreamSynchronize(c->stream));
    }
    return FV_OK;
}


#include "fv_draft_step.hpp"

template int run_step<FV_INST_EL, FV_INST_D>(fv_ctx*, int, StepMode);
template int run_draft_pass<FV_INST_EL, FV_INST_D>(fv_drafter*, const DraftPass&);
template int set_gemm_attrs_d<FV_INST_EL, FV_INST_D>();
template int read_kv_t<FV_INST_EL, FV_INST_D>(fv_ctx*, int, int, int, float*, float*);
#if FV_INST_D == 128
template int tile_upload<FV_INST_EL>(fv_ctx*, int, const GemmPlan&, char*, const void*, size_t, const void*, size_t,
                                     const void*, size_t, int);
#endif
