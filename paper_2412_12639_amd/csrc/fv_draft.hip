// Host side of the drafting-phase entry points declared in include/falcon_verify.h: arena layout of
// the drafter, weight upload, the plan of a phase over a static tree (which rows each pass has, what
// they take in, which row generates which node) and the read-back helpers.  The kernel sequence of a
// pass lives in fv_draft_step.hpp (compiled with the fv_step.hip units).
#include "fv_host.hpp"
#include "fv_draft_kernels.hpp"

#include <algorithm>
#include <cstring>
#include <new>
#include <vector>

namespace {

enum { T_FEAT = 0, T_TOKNODE, T_TOKVAL, T_PRED, T_LPRED, T_BLOCK, T_POS, T_LVL, T_NODEGEN, T_NODERANK, T_EXP };

fv_cfg core_cfg(const fv_cfg& t) {
    fv_cfg c = t;
    c.n_layers = 1;
    c.max_tree = FV_MAX_TREE;
    return c;
}

size_t lstm_stage_elems(const fv_cfg& t) { return (size_t)4 * t.hidden * 2 * t.hidden; }   // lstm0.w_ih, the largest tensor

void make_draft_layout(const fv_cfg& t, int n_wg, DraftLayout& L) {
    const fv_cfg cc = core_cfg(t);
    Layout core;
    make_layout(cc, n_wg, core, false, lstm_stage_elems(t));
    const size_t h = t.hidden, ESZ = core.ESZ, Tpm = FV_MAX_TREE;
    plan_gemm_forms(L.ih0.gm, L.ih0.gd, L.ih0.gp, L.ih0.paired_ok, (int)(4 * h / 32), (int)(2 * h), core.E, n_wg);
    plan_gemm_forms(L.hh.gm, L.hh.gd, L.hh.gp, L.hh.paired_ok, (int)(4 * h / 32), (int)h, core.E, n_wg);
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t r = o; o = rup(o + bytes, 256); return r; };
    L.off_core = take(core.total);
    L.core_bytes = core.total;
    L.off_w[0] = take(L.ih0.gm.tiled_bytes);
    for (int i = 1; i < 4; ++i) L.off_w[i] = take(L.hh.gm.tiled_bytes);
    L.off_bias = take(2 * 4 * h * 4);
    L.off_ones = take(h * 4);
    L.off_xz = take((size_t)L.ih0.gm.Kpad * Tpm * ESZ);
    L.off_xh = take((size_t)L.hh.gm.Kpad * Tpm * ESZ);
    L.off_xprev = take((size_t)L.hh.gm.Kpad * Tpm * ESZ);
    L.off_gin = take(Tpm * 4 * h * 4);
    L.off_grec = take(Tpm * 4 * h * 4);
    L.state_layer_bytes = rup((size_t)(FV_MAX_TREE + 1) * 2 * h * 4, 256);
    L.off_state = take(2 * L.state_layer_bytes);
    L.off_fout = take((size_t)FV_DRAFT_OUT_ROWS * h * 4);
    L.off_top_tok = take((size_t)FV_DRAFT_OUT_ROWS * FV_DRAFT_MMAX * 4);
    L.off_top_val = take((size_t)FV_DRAFT_OUT_ROWS * FV_DRAFT_MMAX * 4);
    L.off_logits = take((size_t)2 * FV_MAX_TREE * core.Vpad * 4);   // a pass writes its padded row count from its first row on
    L.off_node_tok = take(FV_MAX_TREE * 4);
    L.off_tables = take((size_t)FV_DRAFT_TABLES * FV_MAX_TREE * 4);
    L.off_bad = take(256);
    for (GemmPlan* p : {&L.ih0.gm, &L.ih0.gd, &L.ih0.gp, &L.hh.gm, &L.hh.gd, &L.hh.gp}) p->off_tab = take(plan_table_bytes(*p));
    size_t pb = std::max(core.part_bytes, std::max(plan_part_bytes(L.ih0.gm, L.ih0.gd, L.ih0.gp, Tpm), plan_part_bytes(L.hh.gm, L.hh.gd, L.hh.gp, Tpm)));
    L.part_bytes = pb;
    L.off_part = take(pb);
    int ngmax = std::max(L.ih0.gm.n_strips_pad, L.hh.gm.n_strips_pad);
    for (int i = 0; i < GM_COUNT; ++i) ngmax = std::max(ngmax, core.gm[i].n_strips_pad);
    L.ticket_bytes = (size_t)ngmax * 4;
    L.off_tickets = take(L.ticket_bytes);
    L.total = o;
}

int pass_any(fv_drafter* d, const DraftPass& ps) {
    const fv_cfg& cf = d->core->cfg;
    int rc;
    if (cf.dtype == FV_BF16) rc = cf.head_dim == 128 ? run_draft_pass<BF16, 128>(d, ps) : run_draft_pass<BF16, 64>(d, ps);
    else rc = cf.head_dim == 128 ? run_draft_pass<F32, 128>(d, ps) : run_draft_pass<F32, 64>(d, ps);
    if (rc != FV_OK) d->part_dirty = true;   // a pass that stopped half-way may leave partial tiles nobody consumed
    return rc;
}

DraftTables dev_tables(const fv_drafter* d) {
    DraftTables t;
    t.feat_src = d->tab(T_FEAT); t.tok_node = d->tab(T_TOKNODE); t.tok_val = d->tab(T_TOKVAL); t.pred = d->tab(T_PRED);
    t.lpred = d->tab(T_LPRED); t.block = d->tab(T_BLOCK); t.pos = d->tab(T_POS); t.lvl_rows = d->tab(T_LVL);
    t.node_gen = d->tab(T_NODEGEN); t.node_rank = d->tab(T_NODERANK); t.exp_list = d->tab(T_EXP);
    return t;
}

int32_t* htab(fv_drafter* d, int which) { return d->h_tab + (size_t)which * FV_MAX_TREE; }

int upload_tables(fv_drafter* d) {
    HIPCHK(hipMemcpyAsync(d->tab(0), d->h_tab, (size_t)FV_DRAFT_TABLES * FV_MAX_TREE * 4, hipMemcpyHostToDevice, d->core->stream));
    return FV_OK;
}

}  // namespace

extern "C" {

int fv_drafter_workspace_bytes(const fv_cfg* target_cfg, size_t* out_bytes) {
    if (!out_bytes) return FV_E_BAD_ARG;
    int rc = check_cfg(target_cfg);
    if (rc) return rc;
    if (target_cfg->vocab > 32768) return FV_E_BAD_ARG;   // the top-list kernel keeps a row of logits in registers
    DraftLayout L;
    make_draft_layout(*target_cfg, n_workgroups(), L);
    *out_bytes = L.total;
    return FV_OK;
}

int fv_drafter_create(fv_ctx* target, int32_t k, void* dev_arena, size_t arena_bytes, fv_drafter** out) {
    if (!out) return FV_E_BAD_ARG;
    *out = nullptr;
    if (!target || k < 1 || k > FV_DRAFT_KMAX || !dev_arena || ((uintptr_t)dev_arena & 255)) return FV_E_BAD_ARG;
    if (target->cfg.vocab > 32768) return FV_E_BAD_ARG;
    fv_drafter* d = new (std::nothrow) fv_drafter();
    if (!d) return FV_E_BAD_ARG;
    d->target = target;
    d->k = k;
    make_draft_layout(target->cfg, n_workgroups(), d->lay);
    if (arena_bytes < d->lay.total) { delete d; return FV_E_BAD_ARG; }
    d->arena = (char*)dev_arena;
    auto fail = [&](int code) { fv_drafter_destroy(d); return code; };
    const fv_cfg cc = core_cfg(target->cfg);
    int rc = fv_create_ex(&cc, d->arena + d->lay.off_core, d->lay.core_bytes, target->stream, false, lstm_stage_elems(target->cfg), &d->core);
    if (rc) return fail(rc);
    hipStream_t st = d->core->stream;
    // everything outside the core context's part of the arena starts at zero too (states, pad columns, tickets)
    const size_t z0 = d->lay.off_bias;
    if (hipMemsetAsync(d->arena + z0, 0, d->lay.total - z0, st) != hipSuccess) return fail(FV_E_HIP);
    if (hipStreamSynchronize(st) != hipSuccess) return fail(FV_E_HIP);
    {
        std::vector<float> ones(target->cfg.hidden, 1.f);
        if (hipMemcpy(d->arena + d->lay.off_ones, ones.data(), ones.size() * 4, hipMemcpyHostToDevice) != hipSuccess) return fail(FV_E_HIP);
    }
    for (GemmPlan* p : {&d->lay.ih0.gm, &d->lay.ih0.gd, &d->lay.ih0.gp, &d->lay.hh.gm, &d->lay.hh.gd, &d->lay.hh.gp}) {
        std::vector<int> tab;
        p->n_fix = build_split_tables(*p, tab);
        if (tab.size() * 4 > plan_table_bytes(*p)) return fail(FV_E_BAD_ARG);
        if (hipMemcpy(d->arena + p->off_tab, tab.data(), tab.size() * 4, hipMemcpyHostToDevice) != hipSuccess) return fail(FV_E_HIP);
    }
    for (const GemmForms* f : {&d->lay.ih0, &d->lay.hh})
        for (const GemmPlan* q : {&f->gd, &f->gp})
            if ((long long)q->NG * q->NB * (q->G + 1) >= (1LL << 31)) return fail(FV_E_BAD_ARG);
    if (d->lay.part_bytes >= ((size_t)1 << 31)) return fail(FV_E_BAD_ARG);
    d->scr.part = d->at<float>(d->lay.off_part); d->scr.part_bytes = (unsigned)d->lay.part_bytes;
    d->scr.tickets = d->at<int>(d->lay.off_tickets); d->scr.ticket_bytes = d->lay.ticket_bytes;
    d->scr.dirty = &d->part_dirty;
    {   // kernel per LSTM matrix up to 64 rows: the same rule (and the same tuning switch) as the decoder's matrices
        const int base = gemm_kind_from_env();
        d->kind_ih0 = (base == GEMM_PAIRED && !d->lay.ih0.paired_ok) ? GEMM_DIRECT : base;
        d->kind_hh = (base == GEMM_PAIRED && !d->lay.hh.paired_ok) ? GEMM_DIRECT : base;
    }
    if (hipHostMalloc((void**)&d->h_tab, (size_t)FV_DRAFT_TABLES * FV_MAX_TREE * 4, hipHostMallocDefault) != hipSuccess) return fail(FV_E_HIP);
    if (hipHostMalloc((void**)&d->h_out, (FV_MAX_TREE + 64) * 4, hipHostMallocDefault) != hipSuccess) return fail(FV_E_HIP);
    memset(d->h_tab, 0, (size_t)FV_DRAFT_TABLES * FV_MAX_TREE * 4);
    *out = d;
    return FV_OK;
}

void fv_drafter_destroy(fv_drafter* d) {
    if (!d) return;
    if (d->core) fv_destroy(d->core);
    if (d->h_tab) (void)hipHostFree(d->h_tab);
    if (d->h_out) (void)hipHostFree(d->h_out);
    delete d;
}

int fv_drafter_init_weights(fv_drafter* d, const fv_drafter_host_weights* w) {
    if (!d || !w) return FV_E_BAD_ARG;
    for (int l = 0; l < 2; ++l)
        if (!w->lstm_w_ih[l] || !w->lstm_w_hh[l] || !w->lstm_b[l]) return FV_E_BAD_ARG;
    const size_t h = d->core->cfg.hidden;
    int rc = init_layer_weights(d->core, 0, w->wq, w->wk, w->wv, w->wo, w->wg, w->wu, w->wd, w->g_attn, w->g_mlp);
    if (rc) return rc;
    rc = upload_tiled(d->core, d->lay.ih0.gm, d->arena + d->lay.off_w[0], w->lstm_w_ih[0], 4 * h * 2 * h, (int)(4 * h));
    if (rc) return rc;
    rc = upload_tiled(d->core, d->lay.hh.gm, d->arena + d->lay.off_w[1], w->lstm_w_hh[0], 4 * h * h, (int)(4 * h));
    if (rc) return rc;
    rc = upload_tiled(d->core, d->lay.hh.gm, d->arena + d->lay.off_w[2], w->lstm_w_ih[1], 4 * h * h, (int)(4 * h));
    if (rc) return rc;
    rc = upload_tiled(d->core, d->lay.hh.gm, d->arena + d->lay.off_w[3], w->lstm_w_hh[1], 4 * h * h, (int)(4 * h));
    if (rc) return rc;
    for (int l = 0; l < 2; ++l)
        HIPCHK(hipMemcpy(d->arena + d->lay.off_bias + (size_t)l * 4 * h * 4, w->lstm_b[l], 4 * h * 4, hipMemcpyHostToDevice));
    d->core->weights_set = true;
    d->weights_set = true;
    return fv_draft_reset(d);
}

int fv_draft_reset(fv_drafter* d) {
    if (!d) return FV_E_BAD_ARG;
    hipStream_t st = d->core->stream;
    const size_t n = 2 * d->lay.state_layer_bytes / 4;   // all LSTM states, the committed one included
    hipLaunchKernelGGL(k_draft_fill, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, d->at<uint32_t>(d->lay.off_state), 0u, n);
    HIPCHK(hipGetLastError());
    HIPCHK(hipStreamSynchronize(st));
    d->L = d->L0 = 0;
    d->n_chain = d->n_rows = 0;
    return FV_OK;
}

int fv_draft_commit(fv_drafter* d, const int32_t* tokens, const float* dev_features, int32_t n) {
    if (!d || !tokens || !dev_features || n < 1) return FV_E_BAD_ARG;
    if (!d->weights_set || !d->target->weights_set) return FV_E_NO_PREFILL;
    const fv_cfg& cf = d->core->cfg;
    if ((long long)d->L + n > cf.max_seq) return FV_E_CACHE_FULL;
    for (int i = 0; i < n; ++i)
        if (tokens[i] < 0 || tokens[i] >= cf.vocab) return FV_E_TOKEN_RANGE;
    hipStream_t st = d->core->stream;
    float total_ms = 0.f;
    for (int done = 0; done < n;) {
        const int m = std::min(n - done, 64);   // a chain is sequential in the LSTM anyway; 64 rows keep the fast kernels
        if (d->n_chain > 0 && d->k > 1) {       // outputs of the last k-1 committed rows survive the phase that ends
            HistArgs ha;
            ha.fout = d->at<float>(d->lay.off_fout); ha.top_tok = d->at<int32_t>(d->lay.off_top_tok); ha.top_val = d->at<float>(d->lay.off_top_val);
            ha.n_prev = d->n_chain; ha.k = d->k; ha.h = cf.hidden;
            hipLaunchKernelGGL(k_draft_hist, dim3(1), dim3(256), 0, st, ha);
            HIPCHK(hipGetLastError());
        }
        d->L0 = d->L;
        for (int i = 0; i < m; ++i) {
            htab(d, T_FEAT)[i] = -1 - (done + i);
            htab(d, T_TOKNODE)[i] = -1;
            htab(d, T_TOKVAL)[i] = tokens[done + i];
            htab(d, T_PRED)[i] = i - 1;
            htab(d, T_LPRED)[i] = i == 0 ? FV_DRAFT_STATE_COMMITTED : i - 1;
            htab(d, T_BLOCK)[i] = i;           // committed pairs: plain causal order
            htab(d, T_POS)[i] = d->L0 + i;
            htab(d, T_LVL)[i] = i;
        }
        int rc = upload_tables(d);
        if (rc) return rc;
        HIPCHK(hipEventRecord(d->core->ev0, st));
        DraftPass ps;
        ps.r0 = 0; ps.n = m; ps.l0 = 0; ps.lvl_n.assign(m, 1); ps.ext = dev_features;
        rc = pass_any(d, ps);
        if (rc) return rc;
        StateKeepArgs ka;
        ka.state0 = d->state(0); ka.state1 = d->state(1); ka.row = m - 1; ka.h = cf.hidden;
        hipLaunchKernelGGL(k_state_keep, dim3((2 * cf.hidden + 255) / 256), dim3(256), 0, st, ka);
        HIPCHK(hipGetLastError());
        HIPCHK(hipEventRecord(d->core->ev1, st));
        HIPCHK(hipMemcpyAsync(d->h_out + FV_MAX_TREE, d->at<int32_t>(d->lay.off_bad), 8, hipMemcpyDeviceToHost, st));
        HIPCHK(hipStreamSynchronize(st));
        if (d->h_out[FV_MAX_TREE + 1]) { d->part_dirty = true; return FV_E_EXCHANGE_TIMEOUT; }
        float ms = 0.f;
        HIPCHK(hipEventElapsedTime(&ms, d->core->ev0, d->core->ev1));
        total_ms += ms;
        d->L += m;
        d->n_chain = d->n_rows = m;
        done += m;
        if (d->h_out[FV_MAX_TREE]) {
            HIPCHK(hipMemset(d->at<int32_t>(d->lay.off_bad), 0, 4));
            return FV_E_NONFINITE;
        }
    }
    d->last_ms = total_ms;
    return FV_OK;
}

int fv_draft_tree(fv_drafter* d, const int32_t* parent, const int32_t* depth, const int32_t* rank, int32_t n_nodes, int32_t root_token,
                  int32_t* tokens_out) {
    if (!d || !parent || !depth || !rank || !tokens_out || n_nodes < 1) return FV_E_BAD_ARG;
    if (!d->weights_set) return FV_E_NO_PREFILL;
    if (d->n_chain < 1 || d->L < d->k) return FV_E_NO_PREFILL;   // a phase starts with a commit; the root block needs k committed pairs
    if (d->n_rows != d->n_chain) return FV_E_NO_PREFILL;          // one tree per phase
    if (n_nodes > FV_MAX_TREE) return FV_E_TREE_TOO_BIG;
    const fv_cfg& cf = d->core->cfg;
    const int k = d->k, n = n_nodes;
    if (parent[0] != -1) return FV_E_TREE_ORDER;
    for (int i = 1; i < n; ++i)
        if (parent[i] < 0 || parent[i] >= i) return FV_E_TREE_ORDER;
    if (depth[0] != 0) return FV_E_TREE_DEPTH;
    for (int i = 1; i < n; ++i)
        if (depth[i] != depth[parent[i]] + 1) return FV_E_TREE_DEPTH;
    for (int i = 1; i < n; ++i)
        if (rank[i] < 0 || rank[i] >= FV_DRAFT_MMAX || rank[i] >= cf.vocab) return FV_E_BAD_ARG;
    if (root_token < 0 || root_token >= cf.vocab) return FV_E_TOKEN_RANGE;

    // ---- the plan: blocks (one per node at a depth that is a multiple of k and has children), their rows, and for
    // every node the output row and rank that give its token
    std::vector<int> reach(depth, depth + n);
    for (int i = n - 1; i > 0; --i) reach[parent[i]] = std::max(reach[parent[i]], reach[i]);
    int max_depth = 0;
    for (int i = 0; i < n; ++i) max_depth = std::max(max_depth, (int)depth[i]);
    const int n_pass = (max_depth + k - 1) / k;          // the chain pass of the commit counts as the first
    std::vector<std::vector<int>> rows_of(n);            // anchor node -> output row ids of its block
    rows_of[0].resize(k);
    for (int j = 0; j < k; ++j) {                        // root block: the last k committed rows, C[n_chain - 1 + j] of [history, chain]
        const int c = d->n_chain - 1 + j;
        rows_of[0][j] = (c < k - 1) ? FV_MAX_TREE + c : c - (k - 1);
    }
    auto ancestor_at = [&](int i, int dep) { while (depth[i] > dep) i = parent[i]; return i; };
    std::vector<DraftPass> passes;
    int next_row = d->n_chain, lvl_at = 0, exp_at = 0;
    int32_t *t_feat = htab(d, T_FEAT), *t_node = htab(d, T_TOKNODE), *t_val = htab(d, T_TOKVAL), *t_pred = htab(d, T_PRED),
            *t_lpred = htab(d, T_LPRED), *t_block = htab(d, T_BLOCK), *t_pos = htab(d, T_POS), *t_lvl = htab(d, T_LVL),
            *t_gen = htab(d, T_NODEGEN), *t_rank = htab(d, T_NODERANK), *t_exp = htab(d, T_EXP);
    const int base_pos = d->L - 1;                       // position of the root row (the last committed pair)
    for (int p = 1; p < n_pass; ++p) {
        DraftPass ps;
        ps.r0 = next_row; ps.l0 = lvl_at;
        std::vector<std::vector<int>> by_level(k);
        for (int a = 0; a < n; ++a) {
            if (depth[a] != p * k || reach[a] <= depth[a]) continue;
            const int rows = std::min(k, reach[a] - (int)depth[a]);
            const int up = ancestor_at(a, (p - 1) * k);
            if ((int)rows_of[up].size() < k) return FV_E_BAD_ARG;   // cannot happen: a node k levels down has a full block above it
            if (next_row + rows > FV_MAX_TREE) return FV_E_TREE_TOO_BIG;
            for (int j = 0; j < rows; ++j) {
                const int r = next_row++;
                rows_of[a].push_back(r);
                t_feat[r] = rows_of[up][j];
                t_node[r] = ancestor_at(a, (p - 1) * k + j + 1);
                t_val[r] = 0;
                const int before = (j > 0) ? r - 1 : (up == 0 ? d->n_chain - 1 : rows_of[up][k - 1]);
                t_pred[r] = before;
                t_lpred[r] = before;
                t_block[r] = FV_MAX_TREE + a;   // chain rows use their own index as block id
                t_pos[r] = base_pos + (p - 1) * k + j + 1;
                by_level[j].push_back(r - ps.r0);
            }
        }
        ps.n = next_row - ps.r0;
        if (ps.n == 0) return FV_E_BAD_ARG;   // cannot happen: a tree deeper than p*k has a node at depth p*k with children
        for (int j = 0; j < k; ++j) {
            if (by_level[j].empty()) continue;
            ps.lvl_n.push_back((int)by_level[j].size());
            for (int t : by_level[j]) t_lvl[lvl_at++] = t;
        }
        passes.push_back(ps);
    }
    if ((long long)d->L0 + next_row > cf.max_seq) return FV_E_CACHE_FULL;
    // which nodes each pass generates (pass 0: the root block, whose outputs exist since the commit)
    std::vector<std::vector<int>> gen_nodes(n_pass);
    for (int i = 1; i < n; ++i) {
        const int dd = depth[i], p = (dd - 1) / k, j = (dd - 1) % k;
        const int a = ancestor_at(i, p * k);
        if (j >= (int)rows_of[a].size()) return FV_E_BAD_ARG;
        t_gen[i] = rows_of[a][j];
        t_rank[i] = rank[i];
        gen_nodes[p].push_back(i);
    }
    t_gen[0] = 0; t_rank[0] = 0;
    std::vector<std::pair<int, int>> exp_range(n_pass);
    for (int p = 0; p < n_pass; ++p) {
        exp_range[p] = {exp_at, (int)gen_nodes[p].size()};
        for (int i : gen_nodes[p]) t_exp[exp_at++] = i;
    }
    for (int p = 1; p < n_pass; ++p) { passes[p - 1].e0 = exp_range[p].first; passes[p - 1].n_exp = exp_range[p].second; }

    // ---- run: tokens stay on the device between passes
    hipStream_t st = d->core->stream;
    int rc = upload_tables(d);
    if (rc) return rc;
    HIPCHK(hipMemcpyAsync(d->at<int32_t>(d->lay.off_node_tok), &root_token, 4, hipMemcpyHostToDevice, st));
    HIPCHK(hipEventRecord(d->core->ev0, st));
    if (n_pass >= 1 && exp_range[0].second > 0) {
        ExpandArgs ea;
        ea.tab = dev_tables(d); ea.top_tok = d->at<int32_t>(d->lay.off_top_tok); ea.node_tok = d->at<int32_t>(d->lay.off_node_tok);
        ea.e0 = exp_range[0].first; ea.n = exp_range[0].second;
        hipLaunchKernelGGL(k_draft_expand, dim3((ea.n + 255) / 256), dim3(256), 0, st, ea);
        HIPCHK(hipGetLastError());
    }
    for (const DraftPass& ps : passes) {
        rc = pass_any(d, ps);
        if (rc) return rc;
    }
    HIPCHK(hipEventRecord(d->core->ev1, st));
    HIPCHK(hipMemcpyAsync(d->h_out, d->at<int32_t>(d->lay.off_node_tok), (size_t)n * 4, hipMemcpyDeviceToHost, st));
    HIPCHK(hipMemcpyAsync(d->h_out + FV_MAX_TREE, d->at<int32_t>(d->lay.off_bad), 8, hipMemcpyDeviceToHost, st));
    HIPCHK(hipStreamSynchronize(st));
    if (d->h_out[FV_MAX_TREE + 1]) { d->part_dirty = true; return FV_E_EXCHANGE_TIMEOUT; }
    HIPCHK(hipEventElapsedTime(&d->last_ms, d->core->ev0, d->core->ev1));
    d->n_rows = next_row;
    if (d->h_out[FV_MAX_TREE]) {
        HIPCHK(hipMemset(d->at<int32_t>(d->lay.off_bad), 0, 4));
        return FV_E_NONFINITE;
    }
    for (int i = 0; i < n; ++i)
        if (d->h_out[i] < 0 || d->h_out[i] >= cf.vocab) return FV_E_HIP;   // cannot happen with finite logits
    memcpy(tokens_out, d->h_out, (size_t)n * 4);
    return FV_OK;
}

int fv_draft_get_state(fv_drafter* d, int32_t* committed, int32_t* phase_rows, int32_t* chain_rows) {
    if (!d || !committed || !phase_rows || !chain_rows) return FV_E_BAD_ARG;
    *committed = d->L;
    *phase_rows = d->n_rows;
    *chain_rows = d->n_chain;
    return FV_OK;
}

int fv_draft_get_rows(fv_drafter* d, int32_t what, int32_t row0, int32_t n, float* out) {
    if (!d || !out || n < 1 || row0 < 0) return FV_E_BAD_ARG;
    const fv_cfg& cf = d->core->cfg;
    if (what == FV_DRAFT_FEATURES) {
        if (row0 + n > FV_DRAFT_OUT_ROWS) return FV_E_BAD_ARG;
        HIPCHK(hipMemcpy(out, d->at<float>(d->lay.off_fout) + (size_t)row0 * cf.hidden, (size_t)n * cf.hidden * 4, hipMemcpyDeviceToHost));
        return FV_OK;
    }
    if (what == FV_DRAFT_LOGITS) {
        if (row0 + n > d->n_rows) return FV_E_BAD_ARG;
        const size_t Vpad = d->core->lay.Vpad;
        HIPCHK(hipMemcpy2D(out, (size_t)cf.vocab * 4, d->at<float>(d->lay.off_logits) + (size_t)row0 * Vpad, Vpad * 4, (size_t)cf.vocab * 4, n,
                           hipMemcpyDeviceToHost));
        return FV_OK;
    }
    return FV_E_BAD_ARG;
}

int fv_draft_get_top(fv_drafter* d, int32_t row0, int32_t n, int32_t* tokens_out) {
    if (!d || !tokens_out || n < 1 || row0 < 0 || row0 + n > FV_DRAFT_OUT_ROWS) return FV_E_BAD_ARG;
    HIPCHK(hipMemcpy(tokens_out, d->at<int32_t>(d->lay.off_top_tok) + (size_t)row0 * FV_DRAFT_MMAX, (size_t)n * FV_DRAFT_MMAX * 4,
                     hipMemcpyDeviceToHost));
    return FV_OK;
}

int fv_draft_read_kv(fv_drafter* d, int32_t slot0, int32_t n, float* k_out, float* v_out) {
    if (!d) return FV_E_BAD_ARG;
    return fv_read_kv(d->core, 0, slot0, n, k_out, v_out);
}

int fv_draft_last_ms(fv_drafter* d, float* ms) {
    if (!d || !ms) return FV_E_BAD_ARG;
    *ms = d->last_ms;
    return FV_OK;
}

int fv_features_device_ptr(fv_ctx* c, const float** dev_rows) {
    if (!c || !dev_rows) return FV_E_BAD_ARG;
    *dev_rows = c->at<float>(c->lay.off_feat);
    return FV_OK;
}

}  // extern "C"
