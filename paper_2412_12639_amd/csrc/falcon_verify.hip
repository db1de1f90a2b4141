// Host side of the C ABI declared in include/falcon_verify.h: arena layout, weight
// upload, prefill as chain-shaped steps, read-back helpers and timing.  The kernel sequence
// of a step lives in fv_step.hip, compiled once per (element type, head size) pair.
#include "fv_host.hpp"

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

// ---- scratch of fv_verify_tree_noalloc: a file-scope device array, one copy per GPU, held until
// the process ends.  Host code never passes the array's name to a kernel or a HIP call (the name is
// a host-side stand-in, not a device address): the device address is asked for once per device
// with hipGetSymbolAddress and kept in g_static_scratch[].
#define FV_STATIC_SCRATCH_BYTES ((size_t)32 << 20)
#define FV_MAX_DEVICES 64
static __device__ __align__(256) unsigned char scratch[FV_STATIC_SCRATCH_BYTES];
static char* g_static_scratch[FV_MAX_DEVICES];
static bool g_static_dirty[FV_MAX_DEVICES];
static std::mutex g_static_scratch_mu;

// small fill kernel (tickets that must start at zero): a memset node is not what a caller that
// captures this work into a graph wants to see
static __global__ void k_fill_u32(uint32_t* p, uint32_t v, size_t n) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

// plain streaming read (measurement aid, fv_stream_read): one workgroup per compute unit, each wavefront walks its own
// contiguous share with sixteen 16-byte loads per lane in flight
static __global__ __launch_bounds__(256) void k_stream_read(const uint4* p, size_t n16, uint4* sink) {
    const size_t per_wave = n16 / ((size_t)gridDim.x * 4);
    const uint4* q = p + ((size_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * per_wave + (threadIdx.x & 63);
    uint4 acc = make_uint4(0, 0, 0, 0);
    for (size_t i = 0; i + 16 * 64 <= per_wave; i += 16 * 64) {
        uint4 v[16];
#pragma unroll
        for (int k = 0; k < 16; ++k) v[k] = q[i + k * 64];
#pragma unroll
        for (int k = 0; k < 16; ++k) { acc.x ^= v[k].x; acc.y ^= v[k].y; acc.z ^= v[k].z; acc.w ^= v[k].w; }
    }
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9e3779b9u) sink[threadIdx.x] = acc;   // keeps the loads alive; practically never taken
}

// Device address of the current device's copy of `scratch` (looked up once per device).
static int static_scratch_ptr(char** out, bool** dirty) {
    int dev = -1;
    HIPCHK(hipGetDevice(&dev));
    if (dev < 0 || dev >= FV_MAX_DEVICES) return FV_E_BAD_ARG;
    std::lock_guard<std::mutex> lk(g_static_scratch_mu);
    if (!g_static_scratch[dev]) {
        void* ptr = nullptr;
        HIPCHK(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr) return FV_E_HIP;
        g_static_scratch[dev] = (char*)ptr;
    }
    *out = g_static_scratch[dev];
    *dirty = &g_static_dirty[dev];
    return FV_OK;
}

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

// R strips per row group; stage_frags fragments (of 2E columns) per K step of the split (the
// tiled buffer itself is always padded to whole 8-fragment batches)
static void plan_gemm(GemmPlan& p, int n_strips, int K, int E, int n_wg, int R = FV_R, int stage_frags = FV_FRAGS) {
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

// The three forms of one matrix: shared-activation kernel (row groups of FV_R strips), direct kernel
// (one strip per wavefront) and its paired form (two strips per wavefront, half-batch stages).
void plan_gemm_forms(GemmPlan& gm, GemmPlan& gd, GemmPlan& gp, bool& paired_ok, int n_strips, int K, int E, int n_wg) {
    plan_gemm(gm, n_strips, K, E, n_wg);
    plan_gemm(gd, gm.n_strips, gm.K, E, n_wg, 1);
    plan_gemm(gp, gm.n_strips, gm.K, E, n_wg, 2, FV_FRAGS / 2);
    // a full K range must give each streaming wavefront at least three stages, so that no
    // wavefront meets more than two segment ends within one round of three stages
    paired_ok = gp.NB >= 12;
    // Whole row groups per workgroup need no partial-tile exchange at all, but the group counts
    // differ by one between workgroups: worth it only when that idles little of the chip (the
    // LM head: 500 groups of 64 rows over 256 workgroups).  (FV_GEMM_ALIGN=0 / 1 forces it off / on.)
    const char* al = getenv("FV_GEMM_ALIGN");
    for (GemmPlan* q : {&gd, &gp}) {
        if (q->NG < q->G) continue;
        const int per = (q->NG + q->G - 1) / q->G;
        const double idle = (double)((long long)per * q->G - q->NG) / (double)q->NG;
        q->aligned = al ? (!strcmp(al, "1") ? 1 : 0) : (idle <= 0.10 ? 1 : 0);
    }
    for (GemmPlan* q : {&gd, &gp})
        if (q->aligned) q->segmax = (q->NG + q->G - 1) / q->G + 1;
}

// bytes of partial tiles the three forms of one matrix can need at up to T rows (T a multiple of 32)
size_t plan_part_bytes(const GemmPlan& gm, const GemmPlan& gd, const GemmPlan& gp, size_t T) {
    const size_t b = (size_t)gm.G * gm.segmax * FV_R * (T / 32) * 4096;
    const size_t bd = (size_t)gd.G * gd.segmax * 2 * 4096;
    const size_t bp = (size_t)gp.G * gp.segmax * 4 * 4096;
    return std::max(b, std::max(bd, bp));
}

size_t plan_table_bytes(const GemmPlan& p) { return (size_t)(2 * p.G + 1 + 6 * p.NG) * 4 + 16; }

void make_layout(const fv_cfg& c, int n_wg, Layout& L, bool own_head, size_t min_stage_elems) {
    L.E = c.dtype == FV_BF16 ? 8 : 4;
    L.ESZ = c.dtype == FV_BF16 ? 2 : 4;
    L.Tpm = pad_tokens(c.max_tree);
    L.S_pad = (int)rup(c.max_seq, 32);
    const int d = c.head_dim, qd = c.n_q_heads * d, kvd = c.n_kv_heads * d;
    const int ns[GM_COUNT] = {(qd + 2 * kvd) / 32, c.hidden / 32, c.ffn / 16, c.hidden / 32, (c.vocab + 31) / 32};
    const int ks[GM_COUNT] = {c.hidden, qd, c.hidden, c.ffn, c.hidden};
    for (int i = 0; i < GM_COUNT; ++i) plan_gemm_forms(L.gm[i], L.gd[i], L.gp[i], L.paired_ok[i], ns[i], ks[i], L.E, n_wg);
    L.Vpad = L.gm[GM_LM].n_strips * 32;
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t r = o; o = rup(o + bytes, 256); return r; };
    size_t lw = 0;
    for (int i = 0; i < 4; ++i) { L.off_w[i] = lw; lw = rup(lw + L.gm[i].tiled_bytes, 256); }
    L.layer_w_bytes = lw;
    L.off_layers = take(lw * c.n_layers);
    L.off_lm = take(own_head ? L.gm[GM_LM].tiled_bytes : 0);   // a drafter uses the target's head and embedding
    L.off_embed = take(own_head ? (size_t)c.vocab * c.hidden * L.ESZ : 0);
    L.off_gains = take((size_t)(2 * c.n_layers + 1) * c.hidden * 4);
    L.kv_layer_bytes = (size_t)c.n_kv_heads * L.S_pad * d * L.ESZ;
    L.off_k = take(L.kv_layer_bytes * c.n_layers);
    L.off_v = take(L.kv_layer_bytes * c.n_layers);
    const size_t T = L.Tpm;
    L.off_x = take((size_t)c.hidden * T * 4);
    L.off_xb = take((size_t)L.gm[GM_QKV].Kpad * T * L.ESZ);
    L.off_q = take((size_t)qd * T * L.ESZ);
    L.off_qlo = take((size_t)qd * T * L.ESZ);
    L.off_attn = take((size_t)L.gm[GM_O].Kpad * T * L.ESZ);
    L.off_act = take((size_t)L.gm[GM_DN].Kpad * T * L.ESZ);
    L.off_logits = take(T * L.Vpad * 4);
    L.off_ssq = take((size_t)(c.hidden / 32) * T * 4);
    L.off_rinv = take(T * 4);
    size_t pb = 0;
    for (int i = 0; i < GM_COUNT; ++i) pb = std::max(pb, plan_part_bytes(L.gm[i], L.gd[i], L.gp[i], T));
    L.part_bytes = pb;
    L.off_part = take(pb);
    int ngmax = 0;
    for (int i = 0; i < GM_COUNT; ++i) if (L.gm[i].n_strips_pad > ngmax) ngmax = L.gm[i].n_strips_pad;
    L.off_tickets = take((size_t)ngmax * 4);
    for (int i = 0; i < GM_COUNT; ++i) {
        L.gm[i].off_tab = take(plan_table_bytes(L.gm[i]));
        L.gd[i].off_tab = take(plan_table_bytes(L.gd[i]));
        L.gp[i].off_tab = take(plan_table_bytes(L.gp[i]));
    }
    L.off_zeros = take(32768);   // never written after the arena is cleared
    L.off_stepin = take(3 * FV_MAX_TREE * 4);
    L.off_mask = take(FV_MAX_TREE * 4 * 8);
    L.off_pos = take(FV_MAX_TREE * 4);
    L.off_anc = take(FV_MAX_TREE * (FV_CANON_DEPTH + 1));
    L.off_rope = take((size_t)FV_MAX_TREE * (d / 2) * 8);
    L.off_am = take(FV_MAX_TREE * 4);
    L.off_res = take(sizeof(FvResult));
    L.off_feat = take((size_t)FV_MAX_TREE * c.hidden * 4);
    L.off_unif = take((size_t)2 * FV_MAX_TREE * 8);
    L.off_pwork = take((size_t)L.Vpad * 8);
    L.off_kvread = take((size_t)2 * 64 * kvd * 4);
    size_t st = (size_t)(qd + 2 * kvd) * c.hidden;
    const size_t cands[4] = {(size_t)c.hidden * qd, (size_t)2 * c.ffn * c.hidden, (size_t)c.hidden * c.ffn,
                             (size_t)c.vocab * c.hidden};
    for (size_t v : cands) if (v > st && (own_head || v != cands[3])) st = v;
    if (min_stage_elems > st) st = min_stage_elems;
    L.stage_bytes = st * L.ESZ;
    L.off_stage = take(L.stage_bytes);
    // attention key-split partials: at most 8 parts per (head, node block) item, items for 256 rows
    L.off_apart = take((size_t)c.n_q_heads * 8 * 8 * (d / 32 * 1024 + 64) * 4);
    L.off_atick = take((size_t)c.n_q_heads * 8 * 4);
    L.total = o;
}

namespace {

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

template <typename EL>
int run_step_d(fv_ctx* c, int T, StepMode mode) {
    return c->cfg.head_dim == 128 ? run_step<EL, 128>(c, T, mode) : run_step<EL, 64>(c, T, mode);
}
int run_step_any(fv_ctx* c, int T, StepMode mode) {
    const int rc = c->cfg.dtype == FV_BF16 ? run_step_d<BF16>(c, T, mode) : run_step_d<F32>(c, T, mode);
    // a step that did not run to its end may leave partial tiles nobody consumed: have the area cleared before its next use
    if (rc != FV_OK && c->scr && c->scr->dirty) *c->scr->dirty = true;
    return rc;
}

template <typename EL>
int set_gemm_attrs(int head_dim) {
    return head_dim == 128 ? set_gemm_attrs_d<EL, 128>() : set_gemm_attrs_d<EL, 64>();
}

template <typename EL>
int init_layer_t(fv_ctx* c, int l, const void* wq, const void* wk, const void* wv, const void* wo, const void* wg, const void* wu,
                 const void* wd, const float* g_attn, const float* g_mlp) {
    const fv_cfg& cf = c->cfg;
    const Layout& ly = c->lay;
    const size_t h = cf.hidden, qd = (size_t)cf.n_q_heads * cf.head_dim, kvd = (size_t)cf.n_kv_heads * cf.head_dim, F = cf.ffn;
    if (!wq || !wk || !wv || !wo || !wg || !wu || !wd || !g_attn || !g_mlp) return FV_E_BAD_ARG;
    int rc = tile_upload<EL>(c, TILE_QKV, ly.gm[GM_QKV], c->layer_w(l, 0), wq, qd * h, wk, kvd * h, wv, kvd * h, 0);
    if (rc) return rc;
    rc = tile_upload<EL>(c, TILE_NAT, ly.gm[GM_O], c->layer_w(l, 1), wo, h * qd, nullptr, 0, nullptr, 0, (int)h);
    if (rc) return rc;
    rc = tile_upload<EL>(c, TILE_GU, ly.gm[GM_GU], c->layer_w(l, 2), wg, F * h, wu, F * h, nullptr, 0, 0);
    if (rc) return rc;
    rc = tile_upload<EL>(c, TILE_NAT, ly.gm[GM_DN], c->layer_w(l, 3), wd, h * F, nullptr, 0, nullptr, 0, (int)h);
    if (rc) return rc;
    HIPCHK(hipMemcpy(c->gain(2 * l), g_attn, h * 4, hipMemcpyHostToDevice));
    HIPCHK(hipMemcpy(c->gain(2 * l + 1), g_mlp, h * 4, hipMemcpyHostToDevice));
    return FV_OK;
}

template <typename EL>
int init_weights_t(fv_ctx* c, const fv_host_weights* w) {
    const fv_cfg& cf = c->cfg;
    const Layout& ly = c->lay;
    const size_t h = cf.hidden;
    for (int l = 0; l < cf.n_layers; ++l) {
        int rc = init_layer_t<EL>(c, l, w->wq[l], w->wk[l], w->wv[l], w->wo[l], w->wg[l], w->wu[l], w->wd[l], w->g_attn[l], w->g_mlp[l]);
        if (rc) return rc;
    }
    int rc = tile_upload<EL>(c, TILE_NAT, ly.gm[GM_LM], c->arena + ly.off_lm, w->lm_head, (size_t)cf.vocab * h, nullptr, 0, nullptr, 0, cf.vocab);
    if (rc) return rc;
    HIPCHK(hipMemcpy(c->gain(2 * cf.n_layers), w->g_final, h * 4, hipMemcpyHostToDevice));
    HIPCHK(hipMemcpy(c->arena + ly.off_embed, w->embed, (size_t)cf.vocab * h * ly.ESZ, hipMemcpyHostToDevice));
    return FV_OK;
}

}  // namespace

int init_layer_weights(fv_ctx* c, int l, const void* wq, const void* wk, const void* wv, const void* wo, const void* wg,
                       const void* wu, const void* wd, const float* g_attn, const float* g_mlp) {
    return c->cfg.dtype == FV_BF16 ? init_layer_t<BF16>(c, l, wq, wk, wv, wo, wg, wu, wd, g_attn, g_mlp)
                                   : init_layer_t<F32>(c, l, wq, wk, wv, wo, wg, wu, wd, g_attn, g_mlp);
}

int upload_tiled(fv_ctx* c, const GemmPlan& p, char* out, const void* host, size_t n_elems, int N) {
    return c->cfg.dtype == FV_BF16 ? tile_upload<BF16>(c, TILE_NAT, p, out, host, n_elems, nullptr, 0, nullptr, 0, N)
                                   : tile_upload<F32>(c, TILE_NAT, p, out, host, n_elems, nullptr, 0, nullptr, 0, N);
}

int gemm_kind_from_env() {
    const char* e = getenv("FV_GEMM");
    return !e ? GEMM_PAIRED : !strcmp(e, "shared") ? GEMM_SHARED : !strcmp(e, "direct") ? GEMM_DIRECT : GEMM_PAIRED;
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
        case FV_E_NONFINITE: return "non-finite logits";
        case FV_E_EXCHANGE_TIMEOUT: return "a GEMM workgroup waited in vain for another one's partial sums (the context is unusable)";
        case FV_E_SCRATCH_LIMIT: return "beyond the limits of the static scratch (more than 64 nodes, or a shape whose partial tiles exceed it)";
    }
    return "unknown status";
}

int fv_workspace_bytes(const fv_cfg* cfg, size_t* out_bytes) {
    if (!out_bytes) return FV_E_BAD_ARG;
    int rc = check_cfg(cfg);
    if (rc) return rc;
    Layout L;
    make_layout(*cfg, n_workgroups(), L, true, 0);
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
    return fv_create_ex(cfg, dev_arena, arena_bytes, hip_stream, true, 0, out);
}

}  // extern "C"

int fv_create_ex(const fv_cfg* cfg, void* dev_arena, size_t arena_bytes, void* hip_stream, bool own_head, size_t min_stage_elems,
                 fv_ctx** out) {
    if (!out) return FV_E_BAD_ARG;
    *out = nullptr;
    int rc = check_cfg(cfg);
    if (rc) return rc;
    if (!dev_arena || ((uintptr_t)dev_arena & 255)) return FV_E_BAD_ARG;
    fv_ctx* c = new (std::nothrow) fv_ctx();
    if (!c) return FV_E_BAD_ARG;
    c->cfg = *cfg;
    make_layout(*cfg, n_workgroups(), c->lay, own_head, min_stage_elems);
    if (arena_bytes < c->lay.total) { delete c; return FV_E_BAD_ARG; }
    c->arena = (char*)dev_arena;
    c->stream = (hipStream_t)hip_stream;
    {   // GEMM kernel up to 64 tokens.  Default: the paired form wherever its staging slots suffice.
        // FV_GEMM = direct | paired | shared forces one kind; FV_GEMM_PAIRED_SET = bit mask over
        // (QKV, O, gate/up, down, head) restricts the paired form to those matrices (tuning aid).
        const int kind = gemm_kind_from_env();
        const char* m = getenv("FV_GEMM_PAIRED_SET");
        const int mask = m ? atoi(m) : 31;
        for (int i = 0; i < GM_COUNT; ++i) {
            c->kind[i] = kind;
            if (kind == GEMM_PAIRED && (!c->lay.paired_ok[i] || !((mask >> i) & 1))) c->kind[i] = GEMM_DIRECT;
        }
    }
    { const char* e = getenv("FV_GEMM_FIX"); c->gemm_fix = e ? atoi(e) : 1; }
    { const char* e = getenv("FV_ATTN"); c->attn_canon = e && !strcmp(e, "invariant"); }
    { const char* e = getenv("FV_EXCHANGE_TEST"); c->exchange_test = e && !strcmp(e, "timeout"); }
    auto fail = [&](int code) { fv_destroy(c); return code; };
    if (hipHostMalloc((void**)&c->h_in, 3 * FV_MAX_TREE * 4, hipHostMallocDefault) != hipSuccess) return fail(FV_E_HIP);
    if (hipHostMalloc((void**)&c->h_res, sizeof(FvResult), hipHostMallocDefault) != hipSuccess) return fail(FV_E_HIP);
    if (hipHostMalloc((void**)&c->h_unif, 2 * FV_MAX_TREE * 8, hipHostMallocDefault) != hipSuccess) return fail(FV_E_HIP);
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
    {
        const Layout& ly = c->lay;
        int ngmax = 0;
        for (int i = 0; i < GM_COUNT; ++i) if (ly.gm[i].n_strips_pad > ngmax) ngmax = ly.gm[i].n_strips_pad;
        StepScratch& a = c->scr_arena;
        a.part = c->at<float>(ly.off_part); a.part_bytes = (unsigned)ly.part_bytes;
        a.tickets = c->at<int>(ly.off_tickets); a.ticket_bytes = (size_t)ngmax * 4;
        a.apart = c->at<float>(ly.off_apart); a.atick = c->at<int>(ly.off_atick); a.atick_bytes = (size_t)cfg->n_q_heads * 8 * 4;
        a.dirty = &c->arena_part_dirty;
        a.aslots = 32;   // the area holds 8 node blocks x 8 parts per head: 32 triples for each of a 64-row step's two blocks
        c->scr = &c->scr_arena;
        // the same buffers for steps of up to 64 rows (direct and paired GEMM forms, two 32-node attention
        // blocks per head, up to 8 key parts each) inside the static array, if they fit
        size_t pb = 0;
        for (int i = 0; i < GM_COUNT; ++i) {
            const size_t bd = (size_t)ly.gd[i].G * ly.gd[i].segmax * 2 * 4096, bp = (size_t)ly.gp[i].G * ly.gp[i].segmax * 4 * 4096;
            pb = std::max(pb, std::max(bd, bp));
        }
        const size_t ab = (size_t)cfg->n_q_heads * 2 * 8 * (cfg->head_dim / 32 * 1024 + 64) * 4;
        size_t o = 0;
        auto take = [&](size_t bytes) { size_t r = o; o = rup(o + bytes, 256); return r; };
        const size_t o_part = take(pb), o_tick = take(a.ticket_bytes), o_ap = take(ab), o_at = take(a.atick_bytes);
        char* base = nullptr;
        bool* static_dirty = nullptr;
        rc = static_scratch_ptr(&base, &static_dirty);
        if (rc) return fail(rc);
        if (o <= FV_STATIC_SCRATCH_BYTES && pb < ((size_t)1 << 31)) {
            StepScratch& t = c->scr_static;
            t.part = (float*)(base + o_part); t.part_bytes = (unsigned)pb;
            t.tickets = (int*)(base + o_tick); t.ticket_bytes = a.ticket_bytes;
            t.apart = (float*)(base + o_ap); t.atick = (int*)(base + o_at); t.atick_bytes = a.atick_bytes;
            t.aslots = 8;
            t.dirty = static_dirty;
        }
    }
    *out = c;
    return FV_OK;
}

extern "C" {

void fv_destroy(fv_ctx* c) {
    if (!c) return;
    if (c->h_in) (void)hipHostFree(c->h_in);
    if (c->h_res) (void)hipHostFree(c->h_res);
    if (c->h_unif) (void)hipHostFree(c->h_unif);
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
    if (c->h_res->next_token < 0) return FV_E_NONFINITE;   // the last row's logits hold a NaN or an infinity
    c->pending = c->h_res->next_token;
    c->prefilled = true;
    *next_token = c->pending;
    return FV_OK;
}

static int verify_tree_impl(fv_ctx* c, const int32_t* tok, const int32_t* parent, const int32_t* depth, int32_t n,
                            int32_t* accepted_len, int32_t* accepted_tokens, int32_t* next_token, StepMode mode = STEP_VERIFY) {
    memcpy(c->h_in, tok, (size_t)n * 4);
    memcpy(c->h_in + FV_MAX_TREE, parent, (size_t)n * 4);
    memcpy(c->h_in + 2 * FV_MAX_TREE, depth, (size_t)n * 4);
    int rc = run_step_any(c, n, mode);
    if (rc) return rc;
    const FvResult& r = *c->h_res;
    if (r.accepted_len == FV_SCAN_NONFINITE) return FV_E_NONFINITE;
    if (r.accepted_len < 0 || r.accepted_len >= n) return FV_E_HIP;   // cannot happen with a valid tree
    *accepted_len = r.accepted_len;
    for (int j = 0; j < r.accepted_len; ++j) accepted_tokens[j] = r.accepted_tokens[j];
    *next_token = r.next_token;
    c->cur_len += r.accepted_len + 1;
    c->pending = r.next_token;
    return FV_OK;
}

int fv_verify_tree(fv_ctx* c, const int32_t* tok, const int32_t* parent, const int32_t* depth, int32_t n,
                   int32_t* accepted_len, int32_t* accepted_tokens, int32_t* next_token) {
    if (!c || !accepted_len || !accepted_tokens || !next_token) return FV_E_BAD_ARG;
    if (!c->weights_set || !c->prefilled) return FV_E_NO_PREFILL;
    int rc = validate_tree(c->cfg, tok, parent, depth, n, c->pending, c->cur_len, true);
    if (rc) return rc;
    c->scr = &c->scr_arena;
    return verify_tree_impl(c, tok, parent, depth, n, accepted_len, accepted_tokens, next_token);
}

int fv_verify_tree_noalloc(fv_ctx* c, const int32_t* tok, const int32_t* parent, const int32_t* depth, int32_t n,
                           int32_t* accepted_len, int32_t* accepted_tokens, int32_t* next_token) {
    if (!c || !accepted_len || !accepted_tokens || !next_token) return FV_E_BAD_ARG;
    if (!c->weights_set || !c->prefilled) return FV_E_NO_PREFILL;
    int rc = validate_tree(c->cfg, tok, parent, depth, n, c->pending, c->cur_len, true);
    if (rc) return rc;
    // limits of the static scratch: steps of up to 64 rows, and a shape whose partial tiles fit
    if (n > FV_NOALLOC_MAX_NODES || !c->scr_static.part) return FV_E_SCRATCH_LIMIT;
    const StepScratch& t = c->scr_static;
    if (c->attn_canon) {   // the attention's far parts must fit its slots too (the step must compute what fv_verify_tree computes)
        int maxdepth = 0;
        for (int i = 0; i < n; ++i) maxdepth = std::max(maxdepth, (int)depth[i]);
        const int pb = (c->cur_len + maxdepth) >> 5;
        if (maxdepth <= FV_CANON_DEPTH && canon_parts(pb > 0 ? pb - 1 : 0) + 1 > t.aslots) return FV_E_SCRATCH_LIMIT;
    }
    // the array keeps the last call's contents (any context on this GPU): tickets must start at zero
    const size_t nt = t.ticket_bytes / 4, na = t.atick_bytes / 4;
    hipLaunchKernelGGL(k_fill_u32, dim3((unsigned)((nt + 255) / 256)), dim3(256), 0, c->stream, (uint32_t*)t.tickets, 0u, nt);
    hipLaunchKernelGGL(k_fill_u32, dim3((unsigned)((na + 255) / 256)), dim3(256), 0, c->stream, (uint32_t*)t.atick, 0u, na);
    HIPCHK(hipGetLastError());
    const bool prof = c->profiling;
    c->profiling = false;   // per-launch events are created on demand: not in a call that must not allocate
    c->scr = &c->scr_static;
    rc = verify_tree_impl(c, tok, parent, depth, n, accepted_len, accepted_tokens, next_token);
    c->scr = &c->scr_arena;
    c->profiling = prof;
    return rc;
}

int fv_verify_tree_sampled(fv_ctx* c, const int32_t* tok, const int32_t* parent, const int32_t* depth, int32_t n,
                           float temperature, const float* dev_draft_probs, const double* u_accept, const double* u_sample,
                           int32_t* accepted_len, int32_t* accepted_tokens, int32_t* next_token) {
    if (!c || !accepted_len || !accepted_tokens || !next_token || !u_accept || !u_sample) return FV_E_BAD_ARG;
    if (!(temperature > 0.f) || !(temperature < INFINITY)) return FV_E_BAD_ARG;
    if (!c->weights_set || !c->prefilled) return FV_E_NO_PREFILL;
    int rc = validate_tree(c->cfg, tok, parent, depth, n, c->pending, c->cur_len, true);
    if (rc) return rc;
    for (int i = 0; i < n; ++i)   // uniforms in [0, 1]; NaN is refused too
        if (!(u_accept[i] >= 0.0 && u_accept[i] <= 1.0) || !(u_sample[i] >= 0.0 && u_sample[i] <= 1.0)) return FV_E_BAD_ARG;
    memcpy(c->h_unif, u_accept, (size_t)n * 8);
    memcpy(c->h_unif + FV_MAX_TREE, u_sample, (size_t)n * 8);
    c->sample_inv_temperature = 1.0 / (double)temperature;
    c->sample_draft = dev_draft_probs;
    c->scr = &c->scr_arena;
    return verify_tree_impl(c, tok, parent, depth, n, accepted_len, accepted_tokens, next_token, STEP_VERIFY_SAMPLED);
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
    switch (which) {
        case FV_ACT_X: off = ly.off_x; F = cf.hidden; f32 = true; break;
        case FV_ACT_XB: off = ly.off_xb; F = cf.hidden; break;
        case FV_ACT_Q: off = ly.off_q; F = qd; break;
        case FV_ACT_ATTN: off = ly.off_attn; F = qd; break;
        case FV_ACT_FFN: off = ly.off_act; F = cf.ffn; break;
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

int fv_stream_read(fv_ctx* c, int32_t passes, float* gbytes_per_s) {
    if (!c || !gbytes_per_s || passes < 1 || passes > 64) return FV_E_BAD_ARG;
    // the tiled weights are the largest thing in the arena: read them (up to 4 GiB of them) from the start
    size_t bytes = c->lay.off_embed < ((size_t)4 << 30) ? c->lay.off_embed : ((size_t)4 << 30);
    bytes &= ~(size_t)(256 * 4 * 16 * 64 * 16 - 1);   // whole wavefront iterations for 256 workgroups
    if (bytes == 0) return FV_E_BAD_ARG;
    hipLaunchKernelGGL(k_stream_read, dim3(256), dim3(256), 0, c->stream, (const uint4*)c->arena, bytes / 16, c->at<uint4>(c->lay.off_zeros));
    HIPCHK(hipEventRecord(c->ev0, c->stream));
    for (int i = 0; i < passes; ++i)
        hipLaunchKernelGGL(k_stream_read, dim3(256), dim3(256), 0, c->stream, (const uint4*)c->arena, bytes / 16, c->at<uint4>(c->lay.off_zeros));
    HIPCHK(hipGetLastError());
    HIPCHK(hipEventRecord(c->ev1, c->stream));
    HIPCHK(hipStreamSynchronize(c->stream));
    float ms = 0.f;
    HIPCHK(hipEventElapsedTime(&ms, c->ev0, c->ev1));
    *gbytes_per_s = (float)((double)bytes * passes / (ms * 1e-3) / 1e9);
    return FV_OK;
}

int fv_set_step_invariant(fv_ctx* c, int32_t enabled) {
    if (!c || (enabled != 0 && enabled != 1)) return FV_E_BAD_ARG;
    c->attn_canon = enabled != 0;
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
