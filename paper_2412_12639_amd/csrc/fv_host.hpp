// Host-side declarations shared by the translation units of the library: the arena layout,
// the context, and the per-(element type, head size) entry points.  The kernels are compiled
// once per (element type, head size) pair, each pair in a translation unit of its own
// (fv_step.hip), so that the library builds in parallel.
#pragma once
#include "../../include/falcon_verify.h"
#include "fv_internal.h"
#include "fv_types.hpp"
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <vector>

struct BF16;
struct F32;

#define HIPCHK(x)                                                                              \
    do {                                                                                       \
        hipError_t e_ = (x);                                                                   \
        if (e_ != hipSuccess) {                                                                \
            if (getenv("FV_DEBUG")) fprintf(stderr, "falcon_verify: %s -> %s (%s:%d)\n", #x,   \
                                            hipGetErrorString(e_), __FILE__, __LINE__);        \
            return FV_E_HIP;                                                                   \
        }                                                                                      \
    } while (0)

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
    size_t off_x = 0, off_xb = 0, off_q = 0, off_qlo = 0, off_attn = 0, off_act = 0, off_logits = 0;
    size_t off_ssq = 0, off_rinv = 0, off_part = 0, part_bytes = 0, off_tickets = 0;
    size_t off_stepin = 0, off_mask = 0, off_pos = 0, off_anc = 0, off_rope = 0, off_am = 0, off_res = 0;
    size_t off_kvread = 0, off_stage = 0, stage_bytes = 0;
    size_t off_apart = 0, off_atick = 0, off_zeros = 0, off_feat = 0;
    size_t off_unif = 0, off_pwork = 0;   // non-greedy acceptance: uniforms [2][256] fp64, working distribution [Vpad] fp64
    size_t total = 0;
};

inline int pad_tokens(int n) {   // token count padded to 32, 64, 128 or 256
    int tp = 32;
    while (tp < n) tp *= 2;
    return tp;
}


// GEMM kernel used up to 64 tokens (above that always the shared-activation kernel)
enum GemmKind { GEMM_SHARED = 0, GEMM_DIRECT = 1, GEMM_PAIRED = 3 };
enum StepMode { STEP_VERIFY = 0, STEP_PREFILL_MID = 1, STEP_PREFILL_LAST = 2, STEP_VERIFY_SAMPLED = 3 };

// Device memory the kernels of a step use beyond inputs and outputs: stream-K partial tiles and
// their tickets, attention key-split partials and their tickets.
struct StepScratch {
    float* part = nullptr; unsigned part_bytes = 0; int* tickets = nullptr; size_t ticket_bytes = 0;
    bool* dirty = nullptr;   // host flag: the partial area may hold something other than zeros (see launch_gemm)
    float* apart = nullptr; int* atick = nullptr; size_t atick_bytes = 0;
    int aslots = 0;   // key-part triples per (head, 32-row block) item that apart holds for a step of up to 64 rows
};

#define FV_EXCHANGE_SPINS 200000u   // looks at a partial tile that has not arrived before a finisher gives up (~0.3 s)


struct fv_ctx {
    fv_cfg cfg;
    Layout lay;
    StepScratch scr_arena;        // inside the caller's arena
    bool arena_part_dirty = false;
    bool exchange_test = false;   // FV_EXCHANGE_TEST=timeout: contributors leave their partial tiles unmarked, finishers give up after two looks
    StepScratch scr_static;       // inside the library's static device array (steps of up to 64 rows); part == nullptr: does not fit
    const StepScratch* scr = nullptr;   // the one the next step uses
    char* arena = nullptr;
    hipStream_t stream = nullptr;
    bool weights_set = false, prefilled = false;
    int cur_len = 0, pending = -1;
    int last_T = 0, last_Tp = 0, last_L = 0;
    bool last_was_verify = false;
    int32_t* h_in = nullptr;      // pinned [3][256]
    FvResult* h_res = nullptr;    // pinned
    double* h_unif = nullptr;     // pinned [2][256]: u_accept, u_sample of a non-greedy step
    double sample_inv_temperature = 1.0;      // of the non-greedy step being run
    const float* sample_draft = nullptr;      // device [n][vocab] or null
    hipEvent_t ev0 = nullptr, ev1 = nullptr;
    float last_ms = 0.f;
    bool profiling = false;
    int kind[GM_COUNT];       // GemmKind per matrix, used up to 64 tokens
    bool attn_canon = false;     // step-independent attention for verification steps of up to 64 rows (fv_set_step_invariant)
    int gemm_fix = 1;            // 128 / 256 tokens: separate reduction launch for QKV, O and down (FV_GEMM_FIX=0: off, 2: every GEMM)
    std::vector<hipEvent_t> pev;       // event pool for profiling
    std::vector<int> pev_phase;        // phase of each (start, stop) pair
    size_t pev_used = 0;
    float ph_ms[FV_PH_COUNT] = {0, 0, 0, 0};
    int ph_n[FV_PH_COUNT] = {0, 0, 0, 0};

    template <typename T> T* at(size_t off) const { return (T*)(arena + off); }
    char* layer_w(int l, int which) const { return arena + lay.off_layers + (size_t)l * lay.layer_w_bytes + lay.off_w[which]; }
    float* gain(int idx) const { return at<float>(lay.off_gains) + (size_t)idx * cfg.hidden; }   // 2l: attn, 2l+1: mlp, 2NL: final
    char* kc(int l) const { return arena + lay.off_k + (size_t)l * lay.kv_layer_bytes; }
    char* vc(int l) const { return arena + lay.off_v + (size_t)l * lay.kv_layer_bytes; }
};


// ============================================================================ drafting phase
#define FV_DRAFT_STATE_COMMITTED FV_MAX_TREE        // state row of the last committed pair
#define FV_DRAFT_OUT_ROWS (FV_MAX_TREE + FV_DRAFT_KMAX)   // output rows: phase rows + history slots
#define FV_DRAFT_TABLES 11                          // int32 [256] tables of a phase (DraftTables)

struct GemmForms {
    GemmPlan gm, gd, gp;
    bool paired_ok = false;
    const GemmPlan& pick(int kind) const { return kind == GEMM_DIRECT ? gd : kind == GEMM_PAIRED ? gp : gm; }
};

struct DraftLayout {
    GemmForms ih0, hh;                    // [4h x 2h] and [4h x h] (the latter serves lstm0.w_hh, lstm1.w_ih, lstm1.w_hh)
    size_t off_core = 0, core_bytes = 0;  // the decoder block: a one-layer context without head and embedding
    size_t off_w[4] = {0, 0, 0, 0};       // tiled lstm0.w_ih, lstm0.w_hh, lstm1.w_ih, lstm1.w_hh
    size_t off_bias = 0, off_ones = 0;
    size_t off_xz = 0, off_xh = 0, off_xprev = 0, off_gin = 0, off_grec = 0;
    size_t off_state = 0, state_layer_bytes = 0;
    size_t off_fout = 0, off_top_tok = 0, off_top_val = 0, off_logits = 0, off_node_tok = 0, off_tables = 0, off_bad = 0;
    size_t off_part = 0, part_bytes = 0, off_tickets = 0, ticket_bytes = 0;
    size_t total = 0;
};

// one pass of the drafter over phase rows r0 .. r0+n-1
struct DraftPass {
    int r0 = 0, n = 0;
    int l0 = 0;                      // first entry of this pass in lvl_rows
    std::vector<int> lvl_n;          // rows per LSTM level
    int e0 = 0, n_exp = 0;           // tree nodes this pass generates: exp_list[e0 .. e0+n_exp)
    const float* ext = nullptr;      // external features (device), rows addressed by feat_src = -1 - e
};

struct fv_drafter {
    fv_ctx* target = nullptr;
    fv_ctx* core = nullptr;
    DraftLayout lay;
    StepScratch scr;              // partial tiles and tickets large enough for every matrix of the drafter
    bool part_dirty = false;
    char* arena = nullptr;
    int k = 0;
    bool weights_set = false;
    int L = 0;                    // committed pairs whose K/V are in the cache
    int L0 = 0;                   // cache slot of phase row 0
    int n_chain = 0;              // rows of the current phase's chain (0: no phase open)
    int n_rows = 0;               // phase rows so far
    int last_Tp = 0;
    int32_t* h_tab = nullptr;     // pinned [FV_DRAFT_TABLES][256]
    int32_t* h_out = nullptr;     // pinned [256] node tokens + [1] error flag
    float last_ms = 0.f;
    int kind_ih0 = 0, kind_hh = 0;   // GemmKind up to 64 rows

    template <typename T> T* at(size_t off) const { return (T*)(arena + off); }
    float* state(int layer) const { return (float*)(arena + lay.off_state + (size_t)layer * lay.state_layer_bytes); }
    int32_t* tab(int which) const { return (int32_t*)(arena + lay.off_tables) + (size_t)which * FV_MAX_TREE; }
};

// ---- defined in falcon_verify.hip
int check_cfg(const fv_cfg* c);
int n_workgroups();
int gemm_kind_from_env();   // FV_GEMM = paired (default) | direct | shared
void plan_gemm_forms(GemmPlan& gm, GemmPlan& gd, GemmPlan& gp, bool& paired_ok, int n_strips, int K, int E, int n_wg);
size_t plan_part_bytes(const GemmPlan& gm, const GemmPlan& gd, const GemmPlan& gp, size_t T);
size_t plan_table_bytes(const GemmPlan& p);
int build_split_tables(const GemmPlan& p, std::vector<int>& tab);
// own_head = false: no LM head and no embedding table in the arena (a drafter uses the target's);
// min_stage_elems: the upload staging area holds at least that many elements
void make_layout(const fv_cfg& c, int n_wg, Layout& L, bool own_head, size_t min_stage_elems);
int fv_create_ex(const fv_cfg* cfg, void* dev_arena, size_t arena_bytes, void* hip_stream, bool own_head, size_t min_stage_elems,
                 fv_ctx** out);
int init_layer_weights(fv_ctx* c, int l, const void* wq, const void* wk, const void* wv, const void* wo, const void* wg,
                       const void* wu, const void* wd, const float* g_attn, const float* g_mlp);
// upload one row-major [N][K] matrix (p.K = K) and re-tile it for the plan's kernels
int upload_tiled(fv_ctx* c, const GemmPlan& p, char* out, const void* host, size_t n_elems, int N);

// ---- defined in fv_step.hip, instantiated once per (EL, D) pair
// One pass of the decoder over T new rows whose tokens/parent/depth are in c->h_in.
template <typename EL, int D> int run_step(fv_ctx* c, int T, StepMode mode);
// dynamic shared memory limits of the GEMM kernels of this pair
template <typename EL, int D> int set_gemm_attrs_d();
template <typename EL, int D> int read_kv_t(fv_ctx* c, int layer, int slot0, int n, float* k_out, float* v_out);
// upload one weight tensor (up to three host pieces) and re-tile it on the device (independent of D)
// one pass of the drafter (defined in fv_draft_step.hpp, part of the fv_step.hip units)
template <typename EL, int D> int run_draft_pass(fv_drafter* d, const DraftPass& ps);
template <typename EL>
int tile_upload(fv_ctx* c, int kind, const GemmPlan& p, char* out, const void* h0, size_t n0, const void* h1, size_t n1,
                const void* h2, size_t n2, int N);
