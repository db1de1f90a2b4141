// Host side of the C ABI declared in include/falcon_verify.h: arena layout, weight
// upload and tiling, the fixed kernel sequence of one verification step, prefill as
// chain-shaped steps, read-back helpers and timing.
#include "../../include/falcon_verify.h"
#include "fv_kernels.hpp"

#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#define HIPCHK(x)                                                                              \
    do {                                                                                       \
        hipError_t e_ = (x);                                                                   \
        if (e_ != hipSuccess) {                                                                \
            if (getenv("FV_DEBUG")) fprintf(stderr, "falcon_verify: %s -> %s (%s:%d)\n", #x,   \
                                            hipGetErrorString(e_), __FILE__, __LINE__);        \
            return FV_E_HIP;                                                                   \
        }                                                                                      \
    } while (0)

namespace {

inline size_t rup(size_t x, size_t m) { return (x + m - 1) / m * m; }

struct GemmPlan {
    int K = 0, Kpad = 0, NB = 0;
    int n_strips = 0, n_strips_pad = 0, NG = 0;
    int G = 0, segmax = 0;
    int aligned = 0;   // workgroup ranges end on row-group boundaries
    size_t tiled_bytes = 0;
    size_t off_tab = 0;   // device tables: u0[G+1], g0[G], cf[NG], cl[NG], fix[NG][4] (row groups with several contributors:
                          // group, first and last contributor, the first one's segment index)
    int n_fix = 0;        // entries of fix[]
};

enum { GM_QKV = 0, GM_O = 1, GM_GU = 2, GM_DN = 3, GM_LM = 4, GM_COUNT = 5 };

struct Layout {
    int E = 0, ESZ = 0, Tpm = 0, S_pad = 0, Vpad = 0;
    GemmPlan gm[GM_COUNT];    // shared-activation kernel (row groups of FV_R strips)
    GemmPlan gd[GM_COUNT];    // direct kernel (one strip per workgroup at a time), used up to 64 tokens
    GemmPlan gp[GM_COUNT];    // paired form of it (two strips per wavefront, half-batch stages)
    bool paired_ok[GM_COUNT]; // the paired form's two staging slots suffice for this matrix
    size_t layer_w_bytes = 0;        // tiled weights of one layer
    size_t off_w[4] = {0, 0, 0, 0};  // offsets of QKV, O, GU, DN inside a layer
    size_t off_layers = 0, off_lm = 0, off_embed = 0, off_gains = 0;
    size_t off_k = 0, off_v = 0, kv_layer_bytes = 0;
    size_t off_x = 0, off_xb = 0, off_q = 0, off_attn = 0, off_act = 0, off_logits = 0;
    size_t off_ssq = 0, off_rinv = 0, off_part = 0, part_bytes = 0, off_tickets = 0;
    size_t off_stepin = 0, off_mask = 0, off_pos = 0, off_rope = 0, off_am = 0, off_res = 0;
    size_t off_kvread = 0, off_stage = 0, stage_bytes = 0;
    // persistent step kernel: rotating activation slots (one per layer + 1), barrier words, error flag
    size_t off_rot = 0, rot_stride = 0, o_xa = 0, o_xm = 0, o_xba = 0, o_xbm = 0, o_ssqa = 0, o_ssqm = 0, o_q = 0, o_attn = 0, o_act = 0;
    size_t off_bar = 0, off_err = 0, off_tstamp = 0, off_apart = 0, off_atick = 0, off_zeros = 0, off_feat = 0;
    size_t total = 0;
};

int check_cfg(const fv_cfg* c) {
    if (!c) return FV_E_BAD_ARG;
    if (c->dtype != FV_F32 && c->dtype != FV_BF16) return FV_E_BAD_ARG;
    if (c->n_layers < 1 || c->vocab < 1 || c->max_seq < 1) return FV_E_BAD_ARG;
    if (c->head_dim != 64 && c->head_dim != 128) return FV_E_BAD_ARG;
    if (c->hidden < 64 || c->hidden % 64) return FV_E_BAD_ARG;
    if (c->n_q_heads < 1 || c->n_kv_heads < 1 || c->n_q_heads % c->n_kv_heads) return FV_E_BAD_ARG;
    if ((c->n_q_heads * c->head_dim) % 64) return FV_E_BAD_ARG;
    if (c->ffn < 16 || c->ffn % 16) return FV_E_BAD_ARG;
    if (c->max_tree < 1 || c->max_tree > FV_MAX_TREE) return FV_E_BAD_ARG;
    if (!(c->rope_base > 1.f) || !(c->rms_eps > 0.f)) return FV_E_BAD_ARG;
    return FV_OK;
}

int pad_tokens(int n) {   // token count padded to 32, 64, 128 or 256
    int tp = 32;
    while (tp < n) tp *= 2;
    return tp;
}

// R strips per row group; stage_frags fragments (of 2E columns) per K step of the split (the
// tiled buffer itself is always padded to whole 8-fragment batches)
void plan_gemm(GemmPlan& p, int n_strips, int K, int E, int n_wg, int R = FV_R, int stage_frags = FV_FRAGS) {
    const int KB = 16 * E;
    p.K = K;
    p.Kpad = (int)rup(K, KB);
    p.NB = p.Kpad / (2 * E * stage_frags);
    p.n_strips = n_strips;
    p.n_strips_pad = (int)rup(n_strips, FV_R);   // the tiled buffer always holds whole groups of FV_R strips
    p.NG = (R == 1) ? n_strips : p.n_strips_pad / R;
    const long long U = (long long)p.NG * p.NB;
    p.G = (int)(U < n_wg ? U : n_wg);
    const long long per = (U + p.G - 1) / p.G;
    p.segmax = (int)((per + p.NB - 1) / p.NB) + 1;
    p.aligned = 0;
    p.tiled_bytes = (size_t)p.n_strips_pad * (p.Kpad / KB) * FV_FRAGS * 1024;
}

// The stream-K split of one GEMM: workgroup w owns units [u0[w], u0[w+1]) of the (row group,
// K batch) space; g0[w] is its first row group; row group gi is shared by workgroups cf[gi]..cl[gi].
int build_split_tables(const GemmPlan& p, std::vector<int>& tab) {
    const long long U = (long long)p.NG * p.NB;
    const size_t fix_at = ((size_t)2 * p.G + 1 + 2 * p.NG + 3) & ~(size_t)3;   // 16-byte aligned records
    tab.assign(fix_at + 4 * (size_t)p.NG, 0);
    int* u0 = tab.data();
    int* g0 = u0 + p.G + 1;
    int* cf = g0 + p.G;
    int* cl = cf + p.NG;
    int* fix = u0 + fix_at;
    for (int w = 0; w <= p.G; ++w) u0[w] = p.aligned ? (int)((long long)p.NG * w / p.G) * p.NB : (int)(U * w / p.G);
    for (int w = 0; w < p.G; ++w) g0[w] = u0[w] / p.NB;
    for (int gi = 0; gi < p.NG; ++gi) { cf[gi] = p.G; cl[gi] = -1; }
    for (int w = 0; w < p.G; ++w)
        for (int gi = g0[w]; gi <= (u0[w + 1] - 1) / p.NB; ++gi) {
            if (w < cf[gi]) cf[gi] = w;
            if (w > cl[gi]) cl[gi] = w;
        }
    int n_fix = 0;
    for (int gi = 0; gi < p.NG; ++gi)
        if (cl[gi] > cf[gi]) {
            int* rec = fix + 4 * n_fix++;
            rec[0] = gi; rec[1] = cf[gi]; rec[2] = cl[gi]; rec[3] = gi - g0[cf[gi]];
        }
    return n_fix;
}

void make_layout(const fv_cfg& c, int n_wg, Layout& L) {
    L.E = c.dtype == FV_BF16 ? 8 : 4;
    L.ESZ = c.dtype == FV_BF16 ? 2 : 4;
    L.Tpm = pad_tokens(c.max_tree);
    L.S_pad = (int)rup(c.max_seq, 32);
    const int d = c.head_dim, qd = c.n_q_heads * d, kvd = c.n_kv_heads * d;
    plan_gemm(L.gm[GM_QKV], (qd + 2 * kvd) / 32, c.hidden, L.E, n_wg);
    plan_gemm(L.gm[GM_O], c.hidden / 32, qd, L.E, n_wg);
    plan_gemm(L.gm[GM_GU], c.ffn / 16, c.hidden, L.E, n_wg);
    plan_gemm(L.gm[GM_DN], c.hidden / 32, c.ffn, L.E, n_wg);
    plan_gemm(L.gm[GM_LM], (c.vocab + 31) / 32, c.hidden, L.E, n_wg);
    for (int i = 0; i < GM_COUNT; ++i) {
        plan_gemm(L.gd[i], L.gm[i].n_strips, L.gm[i].K, L.E, n_wg, 1);
        plan_gemm(L.gp[i], L.gm[i].n_strips, L.gm[i].K, L.E, n_wg, 2, FV_FRAGS / 2);
        // a full K range must give each of the four wavefronts at least three stages, so that no
        // wavefront meets more than two segment ends within one round of three stages
        L.paired_ok[i] = L.gp[i].NB >= 12;
        // Whole row groups per workgroup need no partial-tile exchange at all, but the group counts
        // differ by one between workgroups: worth it only when that idles little of the chip (the
        // LM head: 500 groups of 64 rows over 256 workgroups).  (FV_GEMM_ALIGN=0 / 1 forces it off / on.)
        const char* al = getenv("FV_GEMM_ALIGN");
        for (GemmPlan* q : {&L.gd[i], &L.gp[i]}) {
            if (q->NG < q->G) continue;
            const int per = (q->NG + q->G - 1) / q->G;
            const double idle = (double)((long long)per * q->G - q->NG) / (double)q->NG;
            q->aligned = al ? (!strcmp(al, "1") ? 1 : 0) : (idle <= 0.10 ? 1 : 0);
        }
        for (GemmPlan* q : {&L.gd[i], &L.gp[i]})
            if (q->aligned) q->segmax = (q->NG + q->G - 1) / q->G + 1;
    }
    L.Vpad = L.gm[GM_LM].n_strips * 32;
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t r = o; o = rup(o + bytes, 256); return r; };
    size_t lw = 0;
    for (int i = 0; i < 4; ++i) { L.off_w[i] = lw; lw = rup(lw + L.gm[i].tiled_bytes, 256); }
    L.layer_w_bytes = lw;
    L.off_layers = take(lw * c.n_layers);
    L.off_lm = take(L.gm[GM_LM].tiled_bytes);
    L.off_embed = take((size_t)c.vocab * c.hidden * L.ESZ);
    L.off_gains = take((size_t)(2 * c.n_layers + 1) * c.hidden * 4);
    L.kv_layer_bytes = (size_t)c.n_kv_heads * L.S_pad * d * L.ESZ;
    L.off_k = take(L.kv_layer_bytes * c.n_layers);
    L.off_v = take(L.kv_layer_bytes * c.n_layers);
    const size_t T = L.Tpm;
    L.off_x = take((size_t)c.hidden * T * 4);
    L.off_xb = take((size_t)L.gm[GM_QKV].Kpad * T * L.ESZ);
    L.off_q = take((size_t)qd * T * L.ESZ);
    L.off_attn = take((size_t)L.gm[GM_O].Kpad * T * L.ESZ);
    L.off_act = take((size_t)L.gm[GM_DN].Kpad * T * L.ESZ);
    L.off_logits = take(T * L.Vpad * 4);
    L.off_ssq = take((size_t)(c.hidden / 32) * T * 4);
    L.off_rinv = take(T * 4);
    size_t pb = 0;
    for (int i = 0; i < GM_COUNT; ++i) {
        const size_t b = (size_t)L.gm[i].G * L.gm[i].segmax * FV_R * (T / 32) * 4096;
        if (b > pb) pb = b;
        const size_t bd = (size_t)L.gd[i].G * L.gd[i].segmax * 2 * 4096;
        if (bd > pb) pb = bd;
        const size_t bp = (size_t)L.gp[i].G * L.gp[i].segmax * 4 * 4096;
        if (bp > pb) pb = bp;
    }
    L.part_bytes = pb;
    L.off_part = take(pb);
    int ngmax = 0;
    for (int i = 0; i < GM_COUNT; ++i) if (L.gm[i].n_strips_pad > ngmax) ngmax = L.gm[i].n_strips_pad;
    L.off_tickets = take((size_t)ngmax * 4);
    for (int i = 0; i < GM_COUNT; ++i) {
        L.gm[i].off_tab = take((size_t)(2 * L.gm[i].G + 1 + 6 * L.gm[i].NG) * 4 + 16);
        L.gd[i].off_tab = take((size_t)(2 * L.gd[i].G + 1 + 6 * L.gd[i].NG) * 4 + 16);
        L.gp[i].off_tab = take((size_t)(2 * L.gp[i].G + 1 + 6 * L.gp[i].NG) * 4 + 16);
    }
    L.off_zeros = take(32768);   // never written after the arena is cleared
    L.off_stepin = take(3 * FV_MAX_TREE * 4);
    L.off_mask = take(FV_MAX_TREE * 4 * 8);
    L.off_pos = take(FV_MAX_TREE * 4);
    L.off_rope = take((size_t)FV_MAX_TREE * (d / 2) * 8);
    L.off_am = take(FV_MAX_TREE * 4);
    L.off_res = take(sizeof(FvResult));
    L.off_feat = take((size_t)FV_MAX_TREE * c.hidden * 4);
    L.off_kvread = take((size_t)2 * 64 * kvd * 4);
    size_t st = (size_t)(qd + 2 * kvd) * c.hidden;
    const size_t cands[4] = {(size_t)c.hidden * qd, (size_t)2 * c.ffn * c.hidden, (size_t)c.hidden * c.ffn,
                             (size_t)c.vocab * c.hidden};
    for (size_t v : cands) if (v > st) st = v;
    L.stage_bytes = st * L.ESZ;
    L.off_stage = take(L.stage_bytes);
    {   // slot of the persistent kernel, sized for 64 tokens
        size_t r = 0;
        auto sub = [&](size_t bytes) { size_t q = r; r = rup(r + bytes, 256); return q; };
        const size_t T64 = 64;
        L.o_xa = sub((size_t)c.hidden * T64 * 4);
        L.o_xm = sub((size_t)c.hidden * T64 * 4);
        L.o_xba = sub((size_t)L.gm[GM_QKV].Kpad * T64 * L.ESZ);
        L.o_xbm = sub((size_t)L.gm[GM_QKV].Kpad * T64 * L.ESZ);
        L.o_ssqa = sub((size_t)(c.hidden / 32) * T64 * 4);
        L.o_ssqm = sub((size_t)(c.hidden / 32) * T64 * 4);
        L.o_q = sub((size_t)qd * T64 * L.ESZ);
        L.o_attn = sub((size_t)L.gm[GM_O].Kpad * T64 * L.ESZ);
        L.o_act = sub((size_t)L.gm[GM_DN].Kpad * T64 * L.ESZ);
        L.rot_stride = r;
        L.off_rot = take(r * (c.n_layers + 1));
        L.off_bar = take((64 + 32 * 256) * 4);
        L.off_err = take(256);
        L.off_tstamp = take(2 * 256 * 16 * 8);
        // attention key-split partials: at most 8 parts per (head, node block) item, items for 256 rows
        L.off_apart = take((size_t)c.n_q_heads * 8 * 8 * (d / 32 * 1024 + 64) * 4);
        L.off_atick = take((size_t)c.n_q_heads * 8 * 4);
    }
    L.total = o;
}

int validate_tree(const fv_cfg& c, const int32_t* tok, const int32_t* parent, const int32_t* depth, int n,
                  int pending, int cur_len, bool check_root) {
    if (!tok || !parent || !depth || n < 1) return FV_E_BAD_ARG;
    if (n > c.max_tree) return FV_E_TREE_TOO_BIG;
    if ((long long)cur_len + n > c.max_seq) return FV_E_CACHE_FULL;
    if (parent[0] != -1) return FV_E_TREE_ORDER;
    for (int i = 1; i < n; ++i)
        if (parent[i] < 0 || parent[i] >= i) return FV_E_TREE_ORDER;
    if (depth[0] != 0) return FV_E_TREE_DEPTH;
    for (int i = 1; i < n; ++i)
        if (depth[i] != depth[parent[i]] + 1) return FV_E_TREE_DEPTH;
    for (int i = 0; i < n; ++i)
        if (tok[i] < 0 || tok[i] >= c.vocab) return FV_E_TOKEN_RANGE;
    if (check_root && tok[0] != pending) return FV_E_ROOT_MISMATCH;
    return FV_OK;
}

}  // namespace

struct fv_ctx {
    fv_cfg cfg;
    Layout lay;
    char* arena = nullptr;
    hipStream_t stream = nullptr;
    bool weights_set = false, prefilled = false;
    int cur_len = 0, pending = -1;
    int last_T = 0, last_Tp = 0, last_L = 0;
    bool last_was_verify = false;
    int32_t* h_in = nullptr;      // pinned [3][256]
    FvResult* h_res = nullptr;    // pinned
    hipEvent_t ev0 = nullptr, ev1 = nullptr;
    float last_ms = 0.f;
    bool profiling = false;
    int kind[GM_COUNT];       // GemmKind per matrix, used up to 64 tokens
    bool persistent_ok = false;  // persistent step kernel asked for (FV_PERSISTENT=1) and cooperative launch available
    int gemm_fix = 1;            // 128 / 256 tokens: separate reduction launch for QKV, O and down (FV_GEMM_FIX=0: off, 2: every GEMM)
    bool last_persistent = false;
    unsigned bar_gen = 0;
    int* h_err = nullptr;        // pinned copy of the persistent kernel's error flag   // FV_GEMM=shared: use the LDS-shared kernel for every token count (tuning)
    std::vector<hipEvent_t> pev;       // event pool for profiling
    std::vector<int> pev_phase;        // phase of each (start, stop) pair
    size_t pev_used = 0;
    float ph_ms[FV_PH_COUNT] = {0, 0, 0, 0, 0};
    int ph_n[FV_PH_COUNT] = {0, 0, 0, 0, 0};

    template <typename T> T* at(size_t off) const { return (T*)(arena + off); }
    char* layer_w(int l, int which) const { return arena + lay.off_layers + (size_t)l * lay.layer_w_bytes + lay.off_w[which]; }
    float* gain(int idx) const { return at<float>(lay.off_gains) + (size_t)idx * cfg.hidden; }   // 2l: attn, 2l+1: mlp, 2NL: final
    char* kc(int l) const { return arena + lay.off_k + (size_t)l * lay.kv_layer_bytes; }
    char* vc(int l) const { return arena + lay.off_v + (size_t)l * lay.kv_layer_bytes; }
};

namespace {

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

template <typename EL, int TB, int D, int EPI>
int launch_gemm_wide_t(fv_ctx* c, const GemmArgs& ga) {
    hipLaunchKernelGGL((k_gemm_wide<EL, TB, D, EPI>), dim3(ga.G), dim3(256), FV_WIDE_SMEM_FLOATS(TB) * 4, c->stream, ga);
    return hipGetLastError() == hipSuccess ? FV_OK : FV_E_HIP;
}

// GEMM kernel used up to 64 tokens (above that always the shared-activation kernel)
enum GemmKind { GEMM_SHARED = 0, GEMM_DIRECT = 1, GEMM_WIDE = 2, GEMM_PAIRED = 3 };

template <typename EL, int TB, int D, int EPI>
int launch_gemm_paired_t(fv_ctx* c, const GemmArgs& ga) {
    hipLaunchKernelGGL((k_gemm_paired<EL, TB, D, EPI>), dim3(ga.G), dim3(256), FV_PAIRED_SMEM_FLOATS(TB) * 4, c->stream, ga);
    return hipGetLastError() == hipSuccess ? FV_OK : FV_E_HIP;
}

template <typename EL, int D, int EPI>
int launch_gemm(fv_ctx* c, int Tp, const GemmArgs& ga, int kind) {
    if (kind == GEMM_DIRECT) return Tp == 32 ? launch_gemm_direct_t<EL, 1, D, EPI>(c, ga) : launch_gemm_direct_t<EL, 2, D, EPI>(c, ga);
    if (kind == GEMM_PAIRED) return Tp == 32 ? launch_gemm_paired_t<EL, 1, D, EPI>(c, ga) : launch_gemm_paired_t<EL, 2, D, EPI>(c, ga);
    if (kind == GEMM_WIDE) return Tp == 32 ? launch_gemm_wide_t<EL, 1, D, EPI>(c, ga) : launch_gemm_wide_t<EL, 2, D, EPI>(c, ga);
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
    HIPCHK(hipFuncSetAttribute((const void*)k_gemm_wide<EL, 1, D, EPI>, hipFuncAttributeMaxDynamicSharedMemorySize, FV_WIDE_SMEM_FLOATS(1) * 4));
    HIPCHK(hipFuncSetAttribute((const void*)k_gemm_wide<EL, 2, D, EPI>, hipFuncAttributeMaxDynamicSharedMemorySize, FV_WIDE_SMEM_FLOATS(2) * 4));
    return FV_OK;
}
template <typename EL, int D>
int set_gemm_attrs_d() {
    int rc = set_gemm_attrs_e<EL, D, EPI_QKV>();
    if (!rc) rc = set_gemm_attrs_e<EL, D, EPI_RESID>();
    if (!rc) rc = set_gemm_attrs_e<EL, D, EPI_SWIGLU>();
    if (!rc) rc = set_gemm_attrs_e<EL, D, EPI_LOGITS>();
    if (!rc) {
        HIPCHK(hipFuncSetAttribute((const void*)k_step_persistent<EL, 1, D, 1>, hipFuncAttributeMaxDynamicSharedMemorySize, FV_PERSIST_SMEM_FLOATS(1, D) * 4));
        HIPCHK(hipFuncSetAttribute((const void*)k_step_persistent<EL, 2, D, 1>, hipFuncAttributeMaxDynamicSharedMemorySize, FV_PERSIST_SMEM_FLOATS(2, D) * 4));
        HIPCHK(hipFuncSetAttribute((const void*)k_step_persistent<EL, 1, D, 2>, hipFuncAttributeMaxDynamicSharedMemorySize, FV_PERSIST_SMEM_FLOATS(1, D) * 4));
        HIPCHK(hipFuncSetAttribute((const void*)k_step_persistent<EL, 2, D, 2>, hipFuncAttributeMaxDynamicSharedMemorySize, FV_PERSIST_SMEM_FLOATS(2, D) * 4));
    }
    return rc;
}
template <typename EL>
int set_gemm_attrs(int head_dim) {
    return head_dim == 128 ? set_gemm_attrs_d<EL, 128>() : set_gemm_attrs_d<EL, 64>();
}

// Key split of the attention: enough workgroups per (head, node block) item to cover the CUs,
// but at least two 32-key blocks each.
int attn_key_split(int items, int n_keys, int n_wg) {
    int ks = n_wg / (items > 0 ? items : 1);
    const int nkb = (n_keys + 31) / 32;
    if (ks > nkb / 2) ks = nkb / 2;
    if (ks > 8) ks = 8;
    if (ks < 1) ks = 1;
    return ks;
}

// All decoder layers in one cooperative launch (see fv_step_persistent.hpp).  Returns FV_OK, or
// a positive value if the launch was refused (the caller then takes the per-GEMM path).
template <typename EL, int D>
int launch_persistent(fv_ctx* c, int T, int Tp, int L) {
    const fv_cfg& cf = c->cfg;
    const Layout& ly = c->lay;
    PersistArgs pa;
    memset(&pa, 0, sizeof(pa));
    pa.n_layers = cf.n_layers; pa.T = T; pa.Tp = Tp; pa.L = L; pa.h = cf.hidden; pa.Hq = cf.n_q_heads; pa.Hkv = cf.n_kv_heads;
    pa.S_pad = ly.S_pad; pa.n_ssq = cf.hidden / 32; pa.inv_h = 1.f / (float)cf.hidden; pa.eps = cf.rms_eps;
    pa.scale = 1.f / std::sqrt((float)D);
    pa.w_layers = c->arena + ly.off_layers; pa.layer_w_bytes = ly.layer_w_bytes;
    for (int i = 0; i < 4; ++i) pa.off_w[i] = ly.off_w[i];
    pa.kc = c->arena + ly.off_k; pa.vc = c->arena + ly.off_v; pa.kv_layer_bytes = ly.kv_layer_bytes;
    pa.gains = c->at<float>(ly.off_gains); pa.rope_cs = c->at<float2>(ly.off_rope); pa.mask = c->at<uint64_t>(ly.off_mask);
    pa.rot = c->arena + ly.off_rot; pa.rot_stride = ly.rot_stride;
    pa.o_xa = ly.o_xa; pa.o_xm = ly.o_xm; pa.o_xba = ly.o_xba; pa.o_xbm = ly.o_xbm; pa.o_ssqa = ly.o_ssqa; pa.o_ssqm = ly.o_ssqm;
    pa.o_q = ly.o_q; pa.o_attn = ly.o_attn; pa.o_act = ly.o_act;
    pa.part = c->at<float>(ly.off_part); pa.part_bytes = (unsigned)ly.part_bytes; pa.tickets = c->at<int>(ly.off_tickets); pa.zeros = c->at<uint4>(ly.off_zeros);
    pa.attn_part = c->at<float>(ly.off_apart); pa.attn_tickets = c->at<int>(ly.off_atick);
    pa.attn_ks = attn_key_split(cf.n_q_heads * (Tp / 32), L + T, 256);
    pa.bar = c->at<unsigned>(ly.off_bar); pa.gen0 = c->bar_gen; pa.err = c->at<int>(ly.off_err);
    pa.tstamp = getenv("FV_PERSIST_TIMING") ? c->at<long long>(ly.off_tstamp) : nullptr;
    pa.ts_phase = getenv("FV_PERSIST_TIMING") ? atoi(getenv("FV_PERSIST_TIMING")) : 0;
    // paired form in the GEMM phases if every layer matrix allows it and it is the selected kind
    bool paired = true;
    for (int i = 0; i < 4; ++i) paired = paired && c->kind[i] == GEMM_PAIRED;
    int grid = 1;
    for (int i = 0; i < 4; ++i) {
        const GemmPlan& p = paired ? ly.gp[i] : ly.gd[i];
        pa.g[i].NG = p.NG; pa.g[i].NB = p.NB; pa.g[i].G = p.G; pa.g[i].segmax = p.segmax; pa.g[i].n_strips = p.n_strips; pa.g[i].aligned = p.aligned;
        pa.g[i].tab = c->at<int>(p.off_tab);
        if (p.G > grid) grid = p.G;
    }
    if (grid > 256) return 1;   // the barrier polls one slot per thread of workgroup 0
    void* args[] = {&pa};
    const void* fn = paired ? ((Tp == 32) ? (const void*)k_step_persistent<EL, 1, D, 2> : (const void*)k_step_persistent<EL, 2, D, 2>)
                            : ((Tp == 32) ? (const void*)k_step_persistent<EL, 1, D, 1> : (const void*)k_step_persistent<EL, 2, D, 1>);
    const unsigned smem = (Tp == 32 ? FV_PERSIST_SMEM_FLOATS(1, D) : FV_PERSIST_SMEM_FLOATS(2, D)) * 4;
    hipError_t e = hipLaunchCooperativeKernel(fn, dim3(grid), dim3(256), args, smem, c->stream);
    if (e != hipSuccess) { (void)hipGetLastError(); return 1; }
    c->bar_gen += 5u * (unsigned)cf.n_layers - 1u;
    return FV_OK;
}

enum StepMode { STEP_VERIFY = 0, STEP_PREFILL_MID = 1, STEP_PREFILL_LAST = 2 };

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

    bool persistent = c->persistent_ok && Tp <= 64;
    HIPCHK(hipMemcpyAsync(c->at<int32_t>(ly.off_stepin), c->h_in, 3 * FV_MAX_TREE * 4, hipMemcpyHostToDevice, st));
    HIPCHK(hipEventRecord(c->ev0, st));
    {
        PhaseTimer pt(c, FV_PH_OTHER);
        IngestArgs ia;
        ia.tok_in = c->at<int32_t>(ly.off_stepin); ia.cap = FV_MAX_TREE; ia.T = T; ia.Tp = Tp; ia.L = L; ia.half_d = D / 2;
        ia.log2_base = std::log2((double)cf.rope_base);
        ia.mask = c->at<uint64_t>(ly.off_mask); ia.pos = c->at<int32_t>(ly.off_pos); ia.rope_cs = c->at<float2>(ly.off_rope);
        hipLaunchKernelGGL(k_ingest, dim3((Tp + 3) / 4), dim3(256), 0, st, ia);
        EmbedArgs ea;
        ea.table = c->at<void>(ly.off_embed); ea.tok = c->at<int32_t>(ly.off_stepin); ea.gain = c->gain(0);
        // the persistent kernel reads layer 0's slot of its rotating buffers
        ea.x = persistent ? (float*)(c->arena + ly.off_rot + ly.o_xa) : c->at<float>(ly.off_x);
        ea.xb = persistent ? (void*)(c->arena + ly.off_rot + ly.o_xba) : c->at<void>(ly.off_xb);
        ea.ssq_part = persistent ? (float*)(c->arena + ly.off_rot + ly.o_ssqa) : c->at<float>(ly.off_ssq);
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
        ga.Wt = (const uint4*)Wt; ga.X = c->at<uint4>(x_off); ga.part = c->at<float>(ly.off_part); ga.part_bytes = (unsigned)ly.part_bytes;
        ga.tickets = c->at<int>(ly.off_tickets); ga.zeros = c->at<uint4>(ly.off_zeros);
        ga.NG = p.NG; ga.NB = p.NB; ga.G = p.G; ga.segmax = p.segmax; ga.aligned = p.aligned;
        ga.tab_u0 = c->at<int>(p.off_tab); ga.tab_g0 = ga.tab_u0 + p.G + 1; ga.tab_cf = ga.tab_g0 + p.G; ga.tab_cl = ga.tab_cf + p.NG;
        ga.fix_groups = (const int4*)(ga.tab_u0 + (((size_t)2 * p.G + 1 + 2 * p.NG + 3) & ~(size_t)3)); ga.n_fix = p.n_fix; ga.rinv_out = c->at<float>(ly.off_rinv);
        ga.T = T; ga.n_strips = p.n_strips;
        ga.ssq_in = c->at<float>(ly.off_ssq); ga.n_ssq = h / 32; ga.inv_h = 1.f / (float)h; ga.eps = cf.rms_eps;
        return ga;
    };

    if (persistent) {
        PhaseTimer pt(c, FV_PH_PERSIST);
        const int rc = launch_persistent<EL, D>(c, T, Tp, L);
        if (rc < 0) return rc;
        if (rc > 0) {   // launch refused: this context takes the per-GEMM path from now on (the embedding is redone below)
            c->persistent_ok = false;
            persistent = false;
            EmbedArgs ea;
            ea.table = c->at<void>(ly.off_embed); ea.tok = c->at<int32_t>(ly.off_stepin); ea.gain = c->gain(0);
            ea.x = c->at<float>(ly.off_x); ea.xb = c->at<void>(ly.off_xb); ea.ssq_part = c->at<float>(ly.off_ssq);
            ea.h = h; ea.T = T; ea.Tp = Tp;
            hipLaunchKernelGGL((k_embed<EL>), dim3(h / 32), dim3(Tp < 64 ? 64 : Tp), 0, st, ea);
            HIPCHK(hipGetLastError());
        }
    }
    const size_t last_slot = ly.off_rot + (size_t)cf.n_layers * ly.rot_stride;
    for (int l = 0; l < cf.n_layers && !persistent; ++l) {
        int rc;
        {   // q, k, v projections of the normalised input, rotary at pos = L + depth, K/V to cache slots L + i
            PhaseTimer pt(c, FV_PH_GEMM);
            GemmArgs ga = gemm_args(GM_QKV, c->layer_w(l, 0), ly.off_xb);
            ga.q_out = c->at<void>(ly.off_q); ga.kcache = c->kc(l); ga.vcache = c->vc(l);
            ga.rope_cs = c->at<float2>(ly.off_rope); ga.Hq = cf.n_q_heads; ga.Hkv = cf.n_kv_heads; ga.L = L; ga.S_pad = ly.S_pad;
            rc = launch_gemm<EL, D, EPI_QKV>(c, Tp, ga, kind_of(GM_QKV));
            if (rc) return rc;
        }
        {
            PhaseTimer pt(c, FV_PH_ATTN);
            AttnArgs aa;
            aa.q = c->at<uint4>(ly.off_q); aa.kc = (const uint4*)c->kc(l); aa.vc = (const uint4*)c->vc(l);
            aa.out = c->at<void>(ly.off_attn); aa.mask = c->at<uint64_t>(ly.off_mask);
            aa.Tp = Tp; aa.T = T; aa.L = L; aa.Hq = cf.n_q_heads; aa.Hkv = cf.n_kv_heads; aa.S_pad = ly.S_pad;
            aa.scale = 1.f / std::sqrt((float)D);
            aa.ks = attn_key_split(cf.n_q_heads * (Tp / 32), L + T, 256);
            aa.part = c->at<float>(ly.off_apart); aa.tickets = c->at<int>(ly.off_atick);
            hipLaunchKernelGGL((k_attn<EL, D>), dim3(cf.n_q_heads * (Tp / 32) * aa.ks), dim3(256), 0, st, aa);
            HIPCHK(hipGetLastError());
        }
        {   // output projection, residual add, statistics + input of the FFN norm
            PhaseTimer pt(c, FV_PH_GEMM);
            GemmArgs ga = gemm_args(GM_O, c->layer_w(l, 1), ly.off_attn);
            ga.x_in = ga.x = c->at<float>(ly.off_x); ga.xb = c->at<void>(ly.off_xb); ga.gain_next = c->gain(2 * l + 1);
            ga.ssq_out = c->at<float>(ly.off_ssq);
            rc = launch_gemm<EL, D, EPI_RESID>(c, Tp, ga, kind_of(GM_O));
            if (rc) return rc;
        }
        {   // gate and up projections, SwiGLU
            PhaseTimer pt(c, FV_PH_GEMM);
            GemmArgs ga = gemm_args(GM_GU, c->layer_w(l, 2), ly.off_xb);
            ga.act = c->at<void>(ly.off_act);
            rc = launch_gemm<EL, D, EPI_SWIGLU>(c, Tp, ga, kind_of(GM_GU));
            if (rc) return rc;
        }
        {   // down projection, residual add, statistics + input of the next norm
            PhaseTimer pt(c, FV_PH_GEMM);
            GemmArgs ga = gemm_args(GM_DN, c->layer_w(l, 3), ly.off_act);
            ga.x_in = ga.x = c->at<float>(ly.off_x); ga.xb = c->at<void>(ly.off_xb);
            ga.gain_next = (l + 1 < cf.n_layers) ? c->gain(2 * (l + 1)) : c->gain(2 * cf.n_layers);
            ga.ssq_out = c->at<float>(ly.off_ssq);
            rc = launch_gemm<EL, D, EPI_RESID>(c, Tp, ga, kind_of(GM_DN));
            if (rc) return rc;
        }
    }

    if (mode != STEP_PREFILL_MID) {
        {
            PhaseTimer pt(c, FV_PH_GEMM);
            GemmArgs ga = gemm_args(GM_LM, c->at<void>(ly.off_lm), persistent ? last_slot + ly.o_xba : ly.off_xb);
            if (persistent) ga.ssq_in = (const float*)(c->arena + last_slot + ly.o_ssqa);
            ga.logits = c->at<float>(ly.off_logits); ga.Vpad = ly.Vpad;
            int rc = launch_gemm<EL, D, EPI_LOGITS>(c, Tp, ga, kind_of(GM_LM));
            if (rc) return rc;
        }
        PhaseTimer pt(c, FV_PH_OTHER);
        ArgmaxArgs am;
        am.logits = c->at<float>(ly.off_logits); am.am = c->at<int32_t>(ly.off_am); am.V = cf.vocab; am.Vpad = ly.Vpad;
        hipLaunchKernelGGL(k_argmax, dim3(T), dim3(256), 0, st, am);
        if (mode == STEP_VERIFY) {
            ScanArgs sa;
            sa.tok_in = c->at<int32_t>(ly.off_stepin); sa.cap = FV_MAX_TREE; sa.T = T;
            sa.mask = c->at<uint64_t>(ly.off_mask); sa.am = c->at<int32_t>(ly.off_am); sa.res = c->at<FvResult>(ly.off_res);
            hipLaunchKernelGGL(k_scan, dim3(1), dim3(256), 0, st, sa);
            CompactArgs ca;
            ca.kcache = c->at<void>(ly.off_k); ca.vcache = c->at<void>(ly.off_v); ca.res = c->at<FvResult>(ly.off_res);
            ca.L = L; ca.S_pad = ly.S_pad;
            hipLaunchKernelGGL((k_compact<EL, D>), dim3(cf.n_layers * cf.n_kv_heads), dim3(D), 0, st, ca);
            // features of the accepted path (what the drafter is given next to the tokens)
            FeatureArgs fa;
            fa.res = c->at<FvResult>(ly.off_res);
            fa.x = persistent ? (const float*)(c->arena + last_slot + ly.o_xa) : c->at<float>(ly.off_x);
            fa.ssq = persistent ? (const float*)(c->arena + last_slot + ly.o_ssqa) : c->at<float>(ly.off_ssq);
            fa.gain = c->gain(2 * cf.n_layers); fa.out = c->at<float>(ly.off_feat);
            fa.h = h; fa.Tp = Tp; fa.inv_h = 1.f / (float)h; fa.eps = cf.rms_eps;
            hipLaunchKernelGGL(k_features, dim3(T), dim3(256), 0, st, fa);
        }
        HIPCHK(hipGetLastError());
    }
    HIPCHK(hipEventRecord(c->ev1, st));
    if (mode == STEP_VERIFY)
        HIPCHK(hipMemcpyAsync(c->h_res, c->at<FvResult>(ly.off_res), sizeof(FvResult), hipMemcpyDeviceToHost, st));
    else if (mode == STEP_PREFILL_LAST)
        HIPCHK(hipMemcpyAsync(&c->h_res->next_token, c->at<int32_t>(ly.off_am) + (T - 1), 4, hipMemcpyDeviceToHost, st));
    if (persistent) HIPCHK(hipMemcpyAsync(c->h_err, c->at<int>(ly.off_err), 4, hipMemcpyDeviceToHost, st));
    HIPCHK(hipStreamSynchronize(st));
    if (persistent && *c->h_err) return FV_E_HIP;   // a grid-barrier wait gave up: results are not valid
    c->last_persistent = persistent;
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
    c->last_was_verify = (mode == STEP_VERIFY);
    return FV_OK;
}

template <typename EL>
int run_step_d(fv_ctx* c, int T, StepMode mode) {
    return c->cfg.head_dim == 128 ? run_step<EL, 128>(c, T, mode) : run_step<EL, 64>(c, T, mode);
}
int run_step_any(fv_ctx* c, int T, StepMode mode) {
    return c->cfg.dtype == FV_BF16 ? run_step_d<BF16>(c, T, mode) : run_step_d<F32>(c, T, mode);
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

template <typename EL>
int init_weights_t(fv_ctx* c, const fv_host_weights* w) {
    const fv_cfg& cf = c->cfg;
    const Layout& ly = c->lay;
    const size_t h = cf.hidden, qd = (size_t)cf.n_q_heads * cf.head_dim, kvd = (size_t)cf.n_kv_heads * cf.head_dim, F = cf.ffn;
    for (int l = 0; l < cf.n_layers; ++l) {
        if (!w->wq[l] || !w->wk[l] || !w->wv[l] || !w->wo[l] || !w->wg[l] || !w->wu[l] || !w->wd[l] || !w->g_attn[l] || !w->g_mlp[l])
            return FV_E_BAD_ARG;
        int rc = tile_upload<EL>(c, TILE_QKV, ly.gm[GM_QKV], c->layer_w(l, 0), w->wq[l], qd * h, w->wk[l], kvd * h, w->wv[l], kvd * h, 0);
        if (rc) return rc;
        rc = tile_upload<EL>(c, TILE_NAT, ly.gm[GM_O], c->layer_w(l, 1), w->wo[l], h * qd, nullptr, 0, nullptr, 0, (int)h);
        if (rc) return rc;
        rc = tile_upload<EL>(c, TILE_GU, ly.gm[GM_GU], c->layer_w(l, 2), w->wg[l], F * h, w->wu[l], F * h, nullptr, 0, 0);
        if (rc) return rc;
        rc = tile_upload<EL>(c, TILE_NAT, ly.gm[GM_DN], c->layer_w(l, 3), w->wd[l], h * F, nullptr, 0, nullptr, 0, (int)h);
        if (rc) return rc;
        HIPCHK(hipMemcpy(c->gain(2 * l), w->g_attn[l], h * 4, hipMemcpyHostToDevice));
        HIPCHK(hipMemcpy(c->gain(2 * l + 1), w->g_mlp[l], h * 4, hipMemcpyHostToDevice));
    }
    int rc = tile_upload<EL>(c, TILE_NAT, ly.gm[GM_LM], c->arena + ly.off_lm, w->lm_head, (size_t)cf.vocab * h, nullptr, 0, nullptr, 0, cf.vocab);
    if (rc) return rc;
    HIPCHK(hipMemcpy(c->gain(2 * cf.n_layers), w->g_final, h * 4, hipMemcpyHostToDevice));
    HIPCHK(hipMemcpy(c->arena + ly.off_embed, w->embed, (size_t)cf.vocab * h * Tr<EL>::ESZ, hipMemcpyHostToDevice));
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

int n_workgroups() {
    // one GEMM workgroup per compute unit; the workspace size must not depend on the
    // machine the size query runs on, so the count is fixed to the MI355X's 256 CUs
    // unless overridden for tuning
    const char* e = getenv("FV_GEMM_WGS");
    int n = e ? atoi(e) : 256;
    if (n < 1) n = 1;
    if (n > 4096) n = 4096;
    return n;
}

}  // namespace

extern "C" {

const char* fv_status_str(int s) {
    switch (s) {
        case FV_OK: return "ok";
        case FV_E_BAD_ARG: return "bad argument";
        case FV_E_TREE_ORDER: return "tree order (parent[0] must be -1, parent[i] in [0, i))";
        case FV_E_TREE_DEPTH: return "depth mismatch";
        case FV_E_TOKEN_RANGE: return "token out of range";
        case FV_E_TREE_TOO_BIG: return "tree larger than max_tree";
        case FV_E_CACHE_FULL: return "KV cache full";
        case FV_E_ROOT_MISMATCH: return "root token is not the pending token";
        case FV_E_NO_PREFILL: return "weights or prefill missing";
        case FV_E_HIP: return "HIP runtime error";
    }
    return "unknown status";
}

int fv_workspace_bytes(const fv_cfg* cfg, size_t* out_bytes) {
    if (!out_bytes) return FV_E_BAD_ARG;
    int rc = check_cfg(cfg);
    if (rc) return rc;
    Layout L;
    make_layout(*cfg, n_workgroups(), L);
    *out_bytes = L.total;
    return FV_OK;
}

int fv_validate_tree(const fv_cfg* cfg, const int32_t* tok, const int32_t* parent, const int32_t* depth, int32_t n,
                     int32_t pending_root, int32_t cur_len) {
    int rc = check_cfg(cfg);
    if (rc) return rc;
    return validate_tree(*cfg, tok, parent, depth, n, pending_root, cur_len, true);
}

int fv_create(const fv_cfg* cfg, void* dev_arena, size_t arena_bytes, void* hip_stream, fv_ctx** out) {
    if (!out) return FV_E_BAD_ARG;
    *out = nullptr;
    int rc = check_cfg(cfg);
    if (rc) return rc;
    if (!dev_arena || ((uintptr_t)dev_arena & 255)) return FV_E_BAD_ARG;
    fv_ctx* c = new (std::nothrow) fv_ctx();
    if (!c) return FV_E_BAD_ARG;
    c->cfg = *cfg;
    make_layout(*cfg, n_workgroups(), c->lay);
    if (arena_bytes < c->lay.total) { delete c; return FV_E_BAD_ARG; }
    c->arena = (char*)dev_arena;
    c->stream = (hipStream_t)hip_stream;
    {   // GEMM kernel up to 64 tokens.  Default: the paired form wherever its staging slots suffice.
        // FV_GEMM = direct | paired | wide | shared forces one kind; FV_GEMM_PAIRED_SET = bit mask over
        // (QKV, O, gate/up, down, head) restricts the paired form to those matrices (tuning aid).
        const char* e = getenv("FV_GEMM");
        const int kind = !e ? GEMM_PAIRED : !strcmp(e, "shared") ? GEMM_SHARED : !strcmp(e, "wide") ? GEMM_WIDE
                       : !strcmp(e, "direct") ? GEMM_DIRECT : GEMM_PAIRED;
        const char* m = getenv("FV_GEMM_PAIRED_SET");
        const int mask = m ? atoi(m) : 31;
        for (int i = 0; i < GM_COUNT; ++i) {
            c->kind[i] = kind;
            if (kind == GEMM_PAIRED && (!c->lay.paired_ok[i] || !((mask >> i) & 1))) c->kind[i] = GEMM_DIRECT;
        }
    }
    // One launch per GEMM is the default: measured on the 7B shape it is ~6% faster per step than
    // the persistent kernel (which wins nothing from its cheaper phase boundaries once 32 layers of
    // rotating activation slots stop fitting the L2s).  FV_PERSISTENT=1 selects the persistent kernel.
    { const char* e = getenv("FV_PERSISTENT"); c->persistent_ok = e && !strcmp(e, "1"); }
    { const char* e = getenv("FV_GEMM_FIX"); c->gemm_fix = e ? atoi(e) : 1; }
    auto fail = [&](int code) { fv_destroy(c); return code; };
    if (hipHostMalloc((void**)&c->h_in, 3 * FV_MAX_TREE * 4, hipHostMallocDefault) != hipSuccess) return fail(FV_E_HIP);
    if (hipHostMalloc((void**)&c->h_res, sizeof(FvResult), hipHostMallocDefault) != hipSuccess) return fail(FV_E_HIP);
    if (hipHostMalloc((void**)&c->h_err, 64, hipHostMallocDefault) != hipSuccess) return fail(FV_E_HIP);
    *c->h_err = 0;
    {
        int dev = 0, coop = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&coop, hipDeviceAttributeCooperativeLaunch, dev) != hipSuccess || !coop)
            c->persistent_ok = false;
    }
    if (hipEventCreate(&c->ev0) != hipSuccess || hipEventCreate(&c->ev1) != hipSuccess) return fail(FV_E_HIP);
    // zero everything except the weights (they are written by fv_init_weights): pad lanes of
    // activations and never-written cache slots must hold finite values
    const size_t z0 = c->lay.off_gains;
    if (hipMemsetAsync(c->arena + z0, 0, c->lay.total - z0, c->stream) != hipSuccess) return fail(FV_E_HIP);
    if (hipStreamSynchronize(c->stream) != hipSuccess) return fail(FV_E_HIP);
    for (int k = 0; k < 3 * GM_COUNT; ++k) {
        GemmPlan& p = (k < GM_COUNT) ? c->lay.gm[k] : (k < 2 * GM_COUNT) ? c->lay.gd[k - GM_COUNT] : c->lay.gp[k - 2 * GM_COUNT];
        std::vector<int> tab;
        p.n_fix = build_split_tables(p, tab);
        if (hipMemcpy(c->arena + p.off_tab, tab.data(), tab.size() * 4, hipMemcpyHostToDevice) != hipSuccess) return fail(FV_E_HIP);
    }
    for (int i = 0; i < GM_COUNT; ++i)   // the direct kernels split their work with 32-bit arithmetic
        for (const GemmPlan* q : {&c->lay.gd[i], &c->lay.gp[i]})
            if ((long long)q->NG * q->NB * (q->G + 1) >= (1LL << 31)) return fail(FV_E_BAD_ARG);
    // the shared-activation kernel addresses the partial tiles with 32-bit byte offsets
    if (c->lay.part_bytes >= ((size_t)1 << 31)) return fail(FV_E_BAD_ARG);
    rc = (cfg->dtype == FV_BF16) ? set_gemm_attrs<BF16>(cfg->head_dim) : set_gemm_attrs<F32>(cfg->head_dim);
    if (rc) return fail(rc);
    *out = c;
    return FV_OK;
}

void fv_destroy(fv_ctx* c) {
    if (!c) return;
    if (c->h_in) (void)hipHostFree(c->h_in);
    if (c->h_res) (void)hipHostFree(c->h_res);
    if (c->h_err) (void)hipHostFree(c->h_err);
    if (c->ev0) (void)hipEventDestroy(c->ev0);
    if (c->ev1) (void)hipEventDestroy(c->ev1);
    for (hipEvent_t e : c->pev) (void)hipEventDestroy(e);
    delete c;
}

int fv_init_weights(fv_ctx* c, const fv_host_weights* w) {
    if (!c || !w || !w->embed || !w->lm_head || !w->g_final || !w->wq || !w->wk || !w->wv || !w->wo || !w->wg || !w->wu ||
        !w->wd || !w->g_attn || !w->g_mlp)
        return FV_E_BAD_ARG;
    int rc = c->cfg.dtype == FV_BF16 ? init_weights_t<BF16>(c, w) : init_weights_t<F32>(c, w);
    if (rc) return rc;
    c->weights_set = true;
    c->prefilled = false;
    return FV_OK;
}

int fv_prefill(fv_ctx* c, const int32_t* tokens, int32_t n, int32_t* next_token) {
    if (!c || !tokens || !next_token || n < 1) return FV_E_BAD_ARG;
    if (!c->weights_set) return FV_E_NO_PREFILL;
    if (n > c->cfg.max_seq) return FV_E_CACHE_FULL;
    for (int i = 0; i < n; ++i)
        if (tokens[i] < 0 || tokens[i] >= c->cfg.vocab) return FV_E_TOKEN_RANGE;
    c->prefilled = false;
    c->cur_len = 0;
    int done = 0;
    while (done < n) {
        const int m = (n - done < c->cfg.max_tree) ? n - done : c->cfg.max_tree;
        for (int i = 0; i < m; ++i) {   // a chain: every token follows the previous one
            c->h_in[i] = tokens[done + i];
            c->h_in[FV_MAX_TREE + i] = i - 1;
            c->h_in[2 * FV_MAX_TREE + i] = i;
        }
        const bool last = done + m == n;
        int rc = run_step_any(c, m, last ? STEP_PREFILL_LAST : STEP_PREFILL_MID);
        if (rc) return rc;
        done += m;
        c->cur_len = done;   // every row of a prompt chunk is kept, already in place
    }
    c->pending = c->h_res->next_token;
    c->prefilled = true;
    *next_token = c->pending;
    return FV_OK;
}

int fv_verify_tree(fv_ctx* c, const int32_t* tok, const int32_t* parent, const int32_t* depth, int32_t n,
                   int32_t* accepted_len, int32_t* accepted_tokens, int32_t* next_token) {
    if (!c || !accepted_len || !accepted_tokens || !next_token) return FV_E_BAD_ARG;
    if (!c->weights_set || !c->prefilled) return FV_E_NO_PREFILL;
    int rc = validate_tree(c->cfg, tok, parent, depth, n, c->pending, c->cur_len, true);
    if (rc) return rc;
    memcpy(c->h_in, tok, (size_t)n * 4);
    memcpy(c->h_in + FV_MAX_TREE, parent, (size_t)n * 4);
    memcpy(c->h_in + 2 * FV_MAX_TREE, depth, (size_t)n * 4);
    rc = run_step_any(c, n, STEP_VERIFY);
    if (rc) return rc;
    const FvResult& r = *c->h_res;
    if (r.accepted_len < 0 || r.accepted_len >= n) return FV_E_HIP;   // cannot happen with a valid tree
    *accepted_len = r.accepted_len;
    for (int j = 0; j < r.accepted_len; ++j) accepted_tokens[j] = r.accepted_tokens[j];
    *next_token = r.next_token;
    c->cur_len += r.accepted_len + 1;
    c->pending = r.next_token;
    return FV_OK;
}

int fv_rollback(fv_ctx* c, int32_t new_len, int32_t pending_root) {
    if (!c) return FV_E_BAD_ARG;
    if (!c->prefilled) return FV_E_NO_PREFILL;
    if (new_len < 0 || new_len > c->cfg.max_seq) return FV_E_BAD_ARG;
    if (pending_root < 0 || pending_root >= c->cfg.vocab) return FV_E_TOKEN_RANGE;
    c->cur_len = new_len;
    c->pending = pending_root;
    return FV_OK;
}

int fv_get_state(fv_ctx* c, int32_t* cur_len, int32_t* pending_root) {
    if (!c || !cur_len || !pending_root) return FV_E_BAD_ARG;
    *cur_len = c->cur_len;
    *pending_root = c->pending;
    return FV_OK;
}

int fv_get_tree_mask(fv_ctx* c, uint64_t* out, int32_t n) {
    if (!c || !out || n < 1 || n > c->last_T) return FV_E_BAD_ARG;
    HIPCHK(hipMemcpy(out, c->at<uint64_t>(c->lay.off_mask), (size_t)n * 32, hipMemcpyDeviceToHost));
    return FV_OK;
}

int fv_get_logits(fv_ctx* c, float* out, int32_t n) {
    if (!c || !out || n < 1 || n > c->last_T) return FV_E_BAD_ARG;
    HIPCHK(hipMemcpy2D(out, (size_t)c->cfg.vocab * 4, c->at<float>(c->lay.off_logits), (size_t)c->lay.Vpad * 4,
                       (size_t)c->cfg.vocab * 4, n, hipMemcpyDeviceToHost));
    return FV_OK;
}

int fv_get_argmax(fv_ctx* c, int32_t* out, int32_t n) {
    if (!c || !out || n < 1 || n > c->last_T) return FV_E_BAD_ARG;
    HIPCHK(hipMemcpy(out, c->at<int32_t>(c->lay.off_am), (size_t)n * 4, hipMemcpyDeviceToHost));
    return FV_OK;
}

int fv_get_kv_moves(fv_ctx* c, int32_t* src, int32_t* dst, int32_t* count) {
    if (!c || !src || !dst || !count || !c->last_was_verify) return FV_E_BAD_ARG;
    const FvResult& r = *c->h_res;
    *count = r.accepted_len + 1;
    for (int j = 0; j <= r.accepted_len; ++j) { src[j] = r.path[j]; dst[j] = c->last_L + j; }
    return FV_OK;
}

int fv_get_features(fv_ctx* c, float* out, int32_t n_rows) {
    if (!c || !out || !c->last_was_verify || n_rows < 1 || n_rows > c->h_res->accepted_len + 1) return FV_E_BAD_ARG;
    HIPCHK(hipMemcpy(out, c->at<float>(c->lay.off_feat), (size_t)n_rows * c->cfg.hidden * 4, hipMemcpyDeviceToHost));
    return FV_OK;
}

int fv_read_kv(fv_ctx* c, int32_t layer, int32_t slot0, int32_t n, float* k_out, float* v_out) {
    if (!c || !k_out || !v_out || layer < 0 || layer >= c->cfg.n_layers || slot0 < 0 || n < 1 ||
        (long long)slot0 + n > c->cfg.max_seq)
        return FV_E_BAD_ARG;
    if (c->cfg.dtype == FV_BF16)
        return c->cfg.head_dim == 128 ? read_kv_t<BF16, 128>(c, layer, slot0, n, k_out, v_out)
                                      : read_kv_t<BF16, 64>(c, layer, slot0, n, k_out, v_out);
    return c->cfg.head_dim == 128 ? read_kv_t<F32, 128>(c, layer, slot0, n, k_out, v_out)
                                  : read_kv_t<F32, 64>(c, layer, slot0, n, k_out, v_out);
}

int fv_debug_read_activation(fv_ctx* c, int32_t which, int32_t n, float* out) {
    if (!c || !out || n < 1 || n > c->last_T) return FV_E_BAD_ARG;
    const fv_cfg& cf = c->cfg;
    const Layout& ly = c->lay;
    const int Tp = c->last_Tp, qd = cf.n_q_heads * cf.head_dim;
    size_t off;
    int F;
    bool f32 = (cf.dtype == FV_F32);
    const bool pe = c->last_persistent;   // the persistent kernel keeps one slot of buffers per layer
    const size_t sl_last = ly.off_rot + (size_t)cf.n_layers * ly.rot_stride, sl_prev = sl_last - ly.rot_stride;
    switch (which) {
        case FV_ACT_X: off = pe ? sl_last + ly.o_xa : ly.off_x; F = cf.hidden; f32 = true; break;
        case FV_ACT_XB: off = pe ? sl_last + ly.o_xba : ly.off_xb; F = cf.hidden; break;
        case FV_ACT_Q: off = pe ? sl_prev + ly.o_q : ly.off_q; F = qd; break;
        case FV_ACT_ATTN: off = pe ? sl_prev + ly.o_attn : ly.off_attn; F = qd; break;
        case FV_ACT_FFN: off = pe ? sl_prev + ly.o_act : ly.off_act; F = cf.ffn; break;
        default: return FV_E_BAD_ARG;
    }
    const int E = f32 ? 4 : 8, esz = f32 ? 4 : 2;
    std::vector<char> buf((size_t)F * Tp * esz);
    HIPCHK(hipMemcpy(buf.data(), c->arena + off, buf.size(), hipMemcpyDeviceToHost));
    for (int t = 0; t < n; ++t)
        for (int f = 0; f < F; ++f) {
            const size_t i = ((size_t)(f / E) * Tp + t) * E + f % E;   // vector-major [F/E][Tp][E]
            float v;
            if (f32) v = ((const float*)buf.data())[i];
            else { uint32_t u = (uint32_t)((const uint16_t*)buf.data())[i] << 16; memcpy(&v, &u, 4); }
            out[(size_t)t * F + f] = v;
        }
    return FV_OK;
}

int fv_debug_persist_timing(fv_ctx* c, long long* out) {
    if (!c || !out) return FV_E_BAD_ARG;
    HIPCHK(hipMemcpy(out, c->at<long long>(c->lay.off_tstamp), 2 * 256 * 16 * 8, hipMemcpyDeviceToHost));
    return FV_OK;
}

int fv_set_profiling(fv_ctx* c, int32_t enabled) {
    if (!c) return FV_E_BAD_ARG;
    c->profiling = enabled != 0;
    return FV_OK;
}

int fv_get_phase_times(fv_ctx* c, float* ms, int32_t* launches) {
    if (!c || !ms || !launches) return FV_E_BAD_ARG;
    for (int i = 0; i < FV_PH_COUNT; ++i) { ms[i] = c->ph_ms[i]; launches[i] = c->ph_n[i]; c->ph_ms[i] = 0.f; c->ph_n[i] = 0; }
    return FV_OK;
}

int fv_last_step_ms(fv_ctx* c, float* ms) {
    if (!c || !ms) return FV_E_BAD_ARG;
    *ms = c->last_ms;
    return FV_OK;
}

}  // extern "C"
