// The kernel sequence of one drafter pass (included by fv_step.hip, one instantiation per
// (element type, head size) pair): input rows -> two LSTM layers, level by level -> the decoder
// block with the relaxed causal mask -> LM head -> top lists.
#pragma once
#include "fv_draft_kernels.hpp"

static DraftTables draft_tables(const fv_drafter* d) {
    DraftTables t;
    t.feat_src = d->tab(0); t.tok_node = d->tab(1); t.tok_val = d->tab(2); t.pred = d->tab(3); t.lpred = d->tab(4);
    t.block = d->tab(5); t.pos = d->tab(6); t.lvl_rows = d->tab(7); t.node_gen = d->tab(8); t.node_rank = d->tab(9);
    t.exp_list = d->tab(10);
    return t;
}

template <typename EL, int D>
int run_draft_pass(fv_drafter* d, const DraftPass& ps) {
    fv_ctx* c = d->core;
    const fv_cfg& cf = c->cfg;
    const Layout& ly = c->lay;
    const DraftLayout& dl = d->lay;
    const int h = cf.hidden, n = ps.n, Tp = pad_tokens(n);
    hipStream_t st = c->stream;
    const DraftTables tab = draft_tables(d);
    constexpr int E = Tr<EL>::E;

    auto kind_for = [&](int tp, int small_kind) { return tp <= 64 ? small_kind : (int)GEMM_SHARED; };
    // a weight multiplication with no norm in front (n_ssq = 0, eps = 1: the per-row factor is rsqrt(1) = 1)
    auto plain_args = [&](const GemmPlan& p, const void* Wt, const void* X, int rows) {
        GemmArgs ga;
        memset(&ga, 0, sizeof(ga));
        ga.Wt = (const uint4*)Wt; ga.X = (const uint4*)X; ga.part = d->scr.part; ga.part_bytes = d->scr.part_bytes;
        ga.tickets = d->scr.tickets; ga.zeros = c->at<uint4>(ly.off_zeros);
        ga.NG = p.NG; ga.NB = p.NB; ga.G = p.G; ga.segmax = p.segmax; ga.aligned = p.aligned;
        ga.tab_u0 = (const int*)(d->arena + p.off_tab); ga.tab_g0 = ga.tab_u0 + p.G + 1; ga.tab_cf = ga.tab_g0 + p.G; ga.tab_cl = ga.tab_cf + p.NG;
        ga.fix_groups = (const int4*)(ga.tab_u0 + (((size_t)2 * p.G + 1 + 2 * p.NG + 3) & ~(size_t)3)); ga.n_fix = p.n_fix;
        ga.rinv_out = c->at<float>(ly.off_rinv);
        ga.T = rows; ga.n_strips = p.n_strips;
        ga.ssq_in = c->at<float>(ly.off_ssq); ga.n_ssq = 0; ga.inv_h = 0.f; ga.eps = 1.f;
        ga.mark = c->exchange_test ? 0u : 1u;
        ga.spin_limit = c->exchange_test ? 2u : FV_EXCHANGE_SPINS;
        ga.fault = d->at<uint32_t>(dl.off_bad) + 1;   // second word of the error slot
        return ga;
    };
    // a matrix of the decoder block (plans and tables of the one-layer context)
    auto core_args = [&](int which, int kind, const void* Wt, size_t x_off, bool with_norm) {
        const GemmPlan& p = (kind == GEMM_DIRECT) ? ly.gd[which] : (kind == GEMM_PAIRED) ? ly.gp[which] : ly.gm[which];
        GemmArgs ga = plain_args(p, Wt, c->at<void>(x_off), n);
        ga.tab_u0 = c->at<int>(p.off_tab); ga.tab_g0 = ga.tab_u0 + p.G + 1; ga.tab_cf = ga.tab_g0 + p.G; ga.tab_cl = ga.tab_cf + p.NG;
        ga.fix_groups = (const int4*)(ga.tab_u0 + (((size_t)2 * p.G + 1 + 2 * p.NG + 3) & ~(size_t)3));
        if (with_norm) { ga.n_ssq = h / 32; ga.inv_h = 1.f / (float)h; ga.eps = cf.rms_eps; }
        return ga;
    };
    auto core_kind = [&](int which) { return (Tp <= 64) ? c->kind[which] : (int)GEMM_SHARED; };
    auto fill = [&](void* p, size_t bytes) {
        hipLaunchKernelGGL(k_draft_fill, dim3((unsigned)((bytes / 4 + 255) / 256)), dim3(256), 0, st, (uint32_t*)p, 0u, bytes / 4);
    };

    if (Tp != d->last_Tp) {   // the row padding changed: what is left in the pad columns is from another layout
        fill(d->at<void>(dl.off_xh), (size_t)h * Tp * Tr<EL>::ESZ);
        fill(c->at<void>(ly.off_x), (size_t)h * Tp * 4);
        fill(c->at<void>(ly.off_xb), (size_t)h * Tp * Tr<EL>::ESZ);
        fill(c->at<void>(ly.off_ssq), (size_t)(h / 32) * Tp * 4);
        d->last_Tp = Tp;
    }
    {
        DraftIngestArgs ia;
        ia.tab = tab; ia.r0 = ps.r0; ia.n = n; ia.Tp = Tp; ia.half_d = D / 2; ia.log2_base = std::log2((double)cf.rope_base);
        ia.mask = c->at<uint64_t>(ly.off_mask); ia.rope_cs = c->at<float2>(ly.off_rope);
        hipLaunchKernelGGL(k_draft_ingest, dim3((Tp + 3) / 4), dim3(256), 0, st, ia);
        DraftInArgs da;
        da.tab = tab; da.fout = d->at<float>(dl.off_fout); da.ext = ps.ext; da.node_tok = d->at<int32_t>(dl.off_node_tok);
        da.table = d->target->arena + d->target->lay.off_embed; da.xz = d->at<void>(dl.off_xz);
        da.r0 = ps.r0; da.n = n; da.Tp = Tp; da.h = h; da.vocab = cf.vocab;
        const size_t items = (size_t)(2 * h / 4) * Tp;
        hipLaunchKernelGGL((k_draft_in<EL>), dim3((unsigned)((items + 255) / 256)), dim3(256), 0, st, da);
        HIPCHK(hipGetLastError());
    }

    // ---- the two LSTM layers: the input multiplication for all rows at once, then level by level the
    // recurrent multiplication and the cell
    for (int layer = 0; layer < 2; ++layer) {
        const GemmForms& fin = layer == 0 ? dl.ih0 : dl.hh;
        {
            const int kind = kind_for(Tp, layer == 0 ? d->kind_ih0 : d->kind_hh);
            const void* X = layer == 0 ? d->at<void>(dl.off_xz) : d->at<void>(dl.off_xh);
            GemmArgs ga = plain_args(fin.pick(kind), d->arena + dl.off_w[2 * layer], X, n);
            ga.logits = d->at<float>(dl.off_gin); ga.Vpad = 4 * h;
            int rc = launch_gemm<EL, D, EPI_LOGITS>(c, Tp, ga, kind, &d->scr);
            if (rc) return rc;
        }
        int l0 = ps.l0;
        for (size_t lv = 0; lv < ps.lvl_n.size(); ++lv) {
            const int nl = ps.lvl_n[lv], Tpl = pad_tokens(nl);
            LstmGatherArgs la;
            la.tab = tab; la.state = d->state(layer); la.xprev = d->at<void>(dl.off_xprev);
            la.r0 = ps.r0; la.l0 = l0; la.n_lvl = nl; la.Tpl = Tpl; la.h = h;
            const size_t items = (size_t)(h / 4) * Tpl;
            hipLaunchKernelGGL((k_lstm_gather<EL>), dim3((unsigned)((items + 255) / 256)), dim3(256), 0, st, la);
            const int kind = kind_for(Tpl, d->kind_hh);
            GemmArgs ga = plain_args(dl.hh.pick(kind), d->arena + dl.off_w[2 * layer + 1], d->at<void>(dl.off_xprev), nl);
            ga.logits = d->at<float>(dl.off_grec); ga.Vpad = 4 * h;
            int rc = launch_gemm<EL, D, EPI_LOGITS>(c, Tpl, ga, kind, &d->scr);
            if (rc) return rc;
            LstmCellArgs ca;
            ca.tab = tab; ca.g_in = d->at<float>(dl.off_gin); ca.g_rec = d->at<float>(dl.off_grec);
            ca.bias = d->at<float>(dl.off_bias) + (size_t)layer * 4 * h; ca.state = d->state(layer);
            ca.xnext = d->at<void>(dl.off_xh); ca.x = c->at<float>(ly.off_x); ca.xb = c->at<void>(ly.off_xb);
            ca.gain = c->gain(0); ca.ssq = c->at<float>(ly.off_ssq);
            ca.r0 = ps.r0; ca.l0 = l0; ca.n_lvl = nl; ca.Tp = Tp; ca.h = h;
            const size_t citems = (size_t)(h / 4) * nl;
            if (layer == 0) hipLaunchKernelGGL((k_lstm_cell<EL, 0>), dim3((unsigned)((citems + 255) / 256)), dim3(256), 0, st, ca);
            else hipLaunchKernelGGL((k_lstm_cell<EL, 1>), dim3((unsigned)((citems + 255) / 256)), dim3(256), 0, st, ca);
            HIPCHK(hipGetLastError());
            l0 += nl;
        }
    }

    // ---- the decoder block over the LSTM output (residual stream x, x * gain and its statistics are in place)
    const int slot0 = d->L0 + ps.r0;   // cache slot of this pass's first row
    {
        GemmArgs ga = core_args(GM_QKV, core_kind(GM_QKV), c->layer_w(0, 0), ly.off_xb, true);
        ga.q_out = c->at<void>(ly.off_q); ga.q_lo_out = c->at<void>(ly.off_qlo); ga.kcache = c->kc(0); ga.vcache = c->vc(0);
        ga.rope_cs = c->at<float2>(ly.off_rope); ga.Hq = cf.n_q_heads; ga.Hkv = cf.n_kv_heads; ga.L = slot0; ga.S_pad = ly.S_pad;
        int rc = launch_gemm<EL, D, EPI_QKV>(c, Tp, ga, core_kind(GM_QKV), &d->scr);
        if (rc) return rc;
    }
    {
        AttnArgs aa;
        aa.q = c->at<uint4>(ly.off_q); aa.q_lo = c->at<uint4>(ly.off_qlo); aa.kc = (const uint4*)c->kc(0); aa.vc = (const uint4*)c->vc(0);
        aa.out = c->at<void>(ly.off_attn); aa.mask = c->at<uint64_t>(ly.off_mask);
        aa.Tp = Tp; aa.T = n; aa.TK = ps.r0 + n; aa.L = d->L0; aa.Hq = cf.n_q_heads; aa.Hkv = cf.n_kv_heads; aa.S_pad = ly.S_pad;
        aa.scale = 1.f / std::sqrt((float)D);
        aa.ks = attn_key_split(cf.n_q_heads * (Tp / 32), d->L0 + ps.r0 + n, 256);
        aa.part = c->scr->apart; aa.tickets = c->scr->atick;
        hipLaunchKernelGGL((k_attn<EL, D>), dim3(cf.n_q_heads * (Tp / 32) * aa.ks), dim3(256), 0, st, aa);
        HIPCHK(hipGetLastError());
    }
    {
        GemmArgs ga = core_args(GM_O, core_kind(GM_O), c->layer_w(0, 1), ly.off_attn, false);
        ga.x_in = ga.x = c->at<float>(ly.off_x); ga.xb = c->at<void>(ly.off_xb); ga.gain_next = c->gain(1);
        ga.ssq_out = c->at<float>(ly.off_ssq);
        int rc = launch_gemm<EL, D, EPI_RESID>(c, Tp, ga, core_kind(GM_O), &d->scr);
        if (rc) return rc;
    }
    {
        GemmArgs ga = core_args(GM_GU, core_kind(GM_GU), c->layer_w(0, 2), ly.off_xb, true);
        ga.act = c->at<void>(ly.off_act);
        int rc = launch_gemm<EL, D, EPI_SWIGLU>(c, Tp, ga, core_kind(GM_GU), &d->scr);
        if (rc) return rc;
    }
    {   // down projection; the block's output is the predicted feature, which the LM head takes as it is (gain 1, no norm)
        GemmArgs ga = core_args(GM_DN, core_kind(GM_DN), c->layer_w(0, 3), ly.off_act, false);
        ga.x_in = ga.x = c->at<float>(ly.off_x); ga.xb = c->at<void>(ly.off_xb); ga.gain_next = d->at<float>(dl.off_ones);
        ga.ssq_out = c->at<float>(ly.off_ssq);
        int rc = launch_gemm<EL, D, EPI_RESID>(c, Tp, ga, core_kind(GM_DN), &d->scr);
        if (rc) return rc;
    }
    {
        DraftOutArgs oa;
        oa.x = c->at<float>(ly.off_x); oa.fout = d->at<float>(dl.off_fout); oa.r0 = ps.r0; oa.n = n; oa.Tp = Tp; oa.h = h;
        hipLaunchKernelGGL(k_draft_out, dim3(n), dim3(256), 0, st, oa);
    }
    {   // the target's LM head on the predicted features; the logits of every phase row are kept (row r at r * Vpad)
        GemmArgs ga = core_args(GM_LM, core_kind(GM_LM), d->target->arena + d->target->lay.off_lm, ly.off_xb, false);
        ga.logits = d->at<float>(dl.off_logits) + (size_t)ps.r0 * ly.Vpad; ga.Vpad = ly.Vpad;
        int rc = launch_gemm<EL, D, EPI_LOGITS>(c, Tp, ga, core_kind(GM_LM), &d->scr);
        if (rc) return rc;
    }
    {
        TopmArgs ta;
        ta.logits = d->at<float>(dl.off_logits) + (size_t)ps.r0 * ly.Vpad; ta.top_tok = d->at<int32_t>(dl.off_top_tok);
        ta.top_val = d->at<float>(dl.off_top_val); ta.bad = d->at<int32_t>(dl.off_bad);
        ta.r0 = ps.r0; ta.n = n; ta.V = cf.vocab; ta.Vpad = ly.Vpad; ta.m = FV_DRAFT_MMAX;
        hipLaunchKernelGGL(k_topm, dim3(n), dim3(FV_TOPM_THREADS), 0, st, ta);   // vocab <= 32768, checked at creation
    }
    if (ps.n_exp > 0) {
        ExpandArgs ea;
        ea.tab = tab; ea.top_tok = d->at<int32_t>(dl.off_top_tok); ea.node_tok = d->at<int32_t>(dl.off_node_tok); ea.e0 = ps.e0; ea.n = ps.n_exp;
        hipLaunchKernelGGL(k_draft_expand, dim3((ps.n_exp + 255) / 256), dim3(256), 0, st, ea);
    }
    HIPCHK(hipGetLastError());
    return FV_OK;
}
