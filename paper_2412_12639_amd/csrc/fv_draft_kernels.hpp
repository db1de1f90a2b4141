// Kernels of the drafting phase (the SAR head of the paper: sections "Framework and Computational
// Process", "Coupled Sequential Glancing Distillation", "Custom-Designed Decoding Tree"; Appendix
// "Tree Structure") that the verification step does not already have: input assembly, the LSTM
// cell, the relaxed causal mask, top-m selection and the expansion of the static tree.  The weight
// multiplications, the attention and the decoder-block epilogues are the verification step's kernels.
//
// Rows of a drafting phase are numbered 0..255 ("phase rows"): first the chain of pairs committed
// since the last phase, then the rows of every tree pass.  A phase row's K/V sits in cache slot
// L0 + row, its 256-bit visibility mask is over phase rows.  "Output rows" are the phase rows plus
// FV_DRAFT_KMAX history slots (ids 256..) that keep the predicted feature and top list of the last
// committed rows of earlier phases.
#pragma once
#include "fv_device.hpp"
#include "fv_types.hpp"

// ---- per-phase tables (device copies of what the host planned from the static tree)
struct DraftTables {
    const int32_t* feat_src;   // [256] phase row -> output row id whose predicted feature it takes in, or -1 - e: row e of the external features
    const int32_t* tok_node;   // [256] phase row -> tree node whose token it takes in, or -1: tok_val
    const int32_t* tok_val;    // [256] token given by the host (committed pairs)
    const int32_t* pred;       // [256] phase row before this one on its path (-1: none; the committed prefix is visible anyway)
    const int32_t* lpred;      // [256] row whose LSTM state it continues (FV_DRAFT_STATE_COMMITTED: the last committed row)
    const int32_t* block;      // [256] block id
    const int32_t* pos;        // [256] rotary position
    const int32_t* lvl_rows;   // [256] rows of each pass grouped by LSTM level (pass-local indices)
    const int32_t* node_gen;   // [256] tree node -> output row id whose top list holds its token
    const int32_t* node_rank;  // [256] tree node -> rank in that list
    const int32_t* exp_list;   // [256] tree nodes grouped by the pass that generates them
};

// ============================================================================ mask, positions, rotary table
// Relaxed causal mask (section "Custom-Designed Decoding Tree"): a row sees its predecessors on its
// path and every row of its own block; the rows of a block are always rows of one pass.
struct DraftIngestArgs {
    DraftTables tab;
    int r0, n, Tp, half_d;
    double log2_base;
    uint64_t* mask;          // [Tp][4]
    float2* rope_cs;         // [Tp][half_d]
};

static __global__ __launch_bounds__(256) void k_draft_ingest(DraftIngestArgs a) {
    const int tid = threadIdx.x;
    const int t0 = blockIdx.x * 4, t1 = (t0 + 4 < a.Tp) ? t0 + 4 : a.Tp;
    for (int t = t0 + tid; t < t1; t += 256) {
        uint64_t m[4] = {0, 0, 0, 0};
        if (t < a.n) {
            const int r = a.r0 + t;
            int j = r, guard = 0;
            while (j >= 0 && j < FV_MAX_TREE && guard++ < FV_MAX_TREE) {   // the host made pred[j] < j; the guard bounds the walk anyway
                m[j >> 6] |= 1ull << (j & 63);
                j = a.tab.pred[j];
            }
            const int b = a.tab.block[r];
            for (int q = a.r0; q < a.r0 + a.n; ++q)
                if (a.tab.block[q] == b) m[q >> 6] |= 1ull << (q & 63);
        }
        for (int w = 0; w < 4; ++w) a.mask[t * 4 + w] = m[w];
    }
    const int n = t1 * a.half_d;
    for (int e = t0 * a.half_d + tid; e < n; e += 256) {
        const int t = e / a.half_d, i = e % a.half_d;
        const int p = (t < a.n) ? a.tab.pos[a.r0 + t] : 0;
        const double inv_freq = exp2(-(double)i / (double)a.half_d * a.log2_base);
        double s, c;
        sincos((double)p * inv_freq, &s, &c);
        a.rope_cs[e] = make_float2((float)c, (float)s);
    }
}

// ============================================================================ input rows
// z = [feature ; embedding of the token one step ahead]  (width 2h), as the vector-major input of
// the first LSTM layer's input multiplication.  Pad columns are zero.
struct DraftInArgs {
    DraftTables tab;
    const float* fout;        // [256 + KMAX][h] predicted features by output row id
    const float* ext;         // external features [..][h] (true features of committed pairs), may be null
    const int32_t* node_tok;  // [256]
    const void* table;        // embedding [V][h]
    void* xz;                 // [2h/E][Tp][E]
    int r0, n, Tp, h, vocab;
};

template <typename EL>
static __global__ __launch_bounds__(256) void k_draft_in(DraftInArgs a) {
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    const int t = (int)(idx % a.Tp);
    const int f0 = (int)(idx / a.Tp) * 4;
    if (f0 >= 2 * a.h) return;
    float v[4] = {0.f, 0.f, 0.f, 0.f};
    if (t < a.n) {
        const int r = a.r0 + t;
        if (f0 < a.h) {
            const int src = a.tab.feat_src[r];
            const float* p = (src >= 0) ? a.fout + (size_t)src * a.h : a.ext + (size_t)(-1 - src) * a.h;
            const float4 x = *(const float4*)(p + f0);
            v[0] = x.x; v[1] = x.y; v[2] = x.z; v[3] = x.w;
        } else {
            const int nd = a.tab.tok_node[r];
            int tok = (nd >= 0) ? a.node_tok[nd] : a.tab.tok_val[r];
            if (tok < 0 || tok >= a.vocab) tok = 0;   // only after a non-finite row, which fails the phase anyway
            const size_t base = (size_t)tok * a.h + (f0 - a.h);
#pragma unroll
            for (int c = 0; c < 4; ++c) v[c] = Tr<EL>::load(a.table, base + c);
        }
    }
    store4_act<EL>(a.xz, a.Tp, f0, t, v[0], v[1], v[2], v[3]);
}

// ============================================================================ LSTM
// State rows: [257][2][h] fp32 per layer (h then c); row 256 is the state after the last committed pair.
// One level = the rows of a pass whose predecessors' states are all known; level rows are listed in
// lvl_rows[l0 .. l0 + n_lvl).

// previous hidden state of every row of a level -> vector-major input of the recurrent multiplication
struct LstmGatherArgs {
    DraftTables tab;
    const float* state;   // this layer's state rows
    void* xprev;          // [h/E][Tpl][E]
    int r0, l0, n_lvl, Tpl, h;
};

template <typename EL>
static __global__ __launch_bounds__(256) void k_lstm_gather(LstmGatherArgs a) {
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    const int i = (int)(idx % a.Tpl);
    const int f0 = (int)(idx / a.Tpl) * 4;
    if (f0 >= a.h) return;
    float4 x = make_float4(0.f, 0.f, 0.f, 0.f);
    if (i < a.n_lvl) {
        const int r = a.r0 + a.tab.lvl_rows[a.l0 + i];
        x = *(const float4*)(a.state + ((size_t)a.tab.lpred[r] * 2) * a.h + f0);
    }
    store4_act<EL>(a.xprev, a.Tpl, f0, i, x.x, x.y, x.z, x.w);
}

// gates = G_in[row] + G_rec[level row] + bias (rows ordered input, forget, cell, output);
// c' = sigmoid(f) c + sigmoid(i) tanh(g);  h' = sigmoid(o) tanh(c').
// LAYER 0: h' also becomes the row's column of the second layer's input.
// LAYER 1: h' is the decoder block's residual stream x; also x * gain (the un-normalised input of the
// q/k/v multiplication) and the per-strip sums of squares of x.
struct LstmCellArgs {
    DraftTables tab;
    const float* g_in;    // [Tp][4h]
    const float* g_rec;   // [Tpl][4h]
    const float* bias;    // [4h]
    float* state;         // this layer's state rows
    void* xnext;          // LAYER 0: [h/E][Tp][E]
    float* x;             // LAYER 1: [h/4][Tp][4]
    void* xb;             // LAYER 1: [h/E][Tp][E]
    const float* gain;    // LAYER 1: [h]
    float* ssq;           // LAYER 1: [h/32][Tp]
    int r0, l0, n_lvl, Tp, h;
};

__device__ __forceinline__ float fv_sigmoid(float x) { return 1.f / (1.f + expf(-x)); }

template <typename EL, int LAYER>
static __global__ __launch_bounds__(256) void k_lstm_cell(LstmCellArgs a) {
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    const int q = a.h / 4;                 // 4-feature groups per row; 8 consecutive lanes share a 32-feature strip
    const int i = (int)(idx / q);
    const int f0 = (int)(idx % q) * 4;
    if (i >= a.n_lvl) return;              // whole strips leave together: h is a multiple of 64
    const int t = a.tab.lvl_rows[a.l0 + i];
    const int r = a.r0 + t;
    const size_t H = a.h;
    const float* gi = a.g_in + (size_t)t * 4 * H;
    const float* gr = a.g_rec + (size_t)i * 4 * H;
    float4 g[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const float4 u = *(const float4*)(gi + k * H + f0), w = *(const float4*)(gr + k * H + f0), b = *(const float4*)(a.bias + k * H + f0);
        g[k] = make_float4(u.x + w.x + b.x, u.y + w.y + b.y, u.z + w.z + b.z, u.w + w.w + b.w);
    }
    const float4 cp = *(const float4*)(a.state + ((size_t)a.tab.lpred[r] * 2 + 1) * H + f0);
    const float gin[4] = {g[0].x, g[0].y, g[0].z, g[0].w}, gf[4] = {g[1].x, g[1].y, g[1].z, g[1].w};
    const float gg[4] = {g[2].x, g[2].y, g[2].z, g[2].w}, go[4] = {g[3].x, g[3].y, g[3].z, g[3].w};
    const float cprev[4] = {cp.x, cp.y, cp.z, cp.w};
    float hn[4], cn[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        cn[c] = fv_sigmoid(gf[c]) * cprev[c] + fv_sigmoid(gin[c]) * tanhf(gg[c]);
        hn[c] = fv_sigmoid(go[c]) * tanhf(cn[c]);
    }
    *(float4*)(a.state + ((size_t)r * 2) * H + f0) = make_float4(hn[0], hn[1], hn[2], hn[3]);
    *(float4*)(a.state + ((size_t)r * 2 + 1) * H + f0) = make_float4(cn[0], cn[1], cn[2], cn[3]);
    if constexpr (LAYER == 0) {
        store4_act<EL>(a.xnext, a.Tp, f0, t, hn[0], hn[1], hn[2], hn[3]);
    } else {
        ((float4*)a.x)[(size_t)(f0 >> 2) * a.Tp + t] = make_float4(hn[0], hn[1], hn[2], hn[3]);
        const float4 gn = *(const float4*)(a.gain + f0);
        store4_act<EL>(a.xb, a.Tp, f0, t, hn[0] * gn.x, hn[1] * gn.y, hn[2] * gn.z, hn[3] * gn.w);
        float ssq = hn[0] * hn[0] + hn[1] * hn[1] + hn[2] * hn[2] + hn[3] * hn[3];
        ssq += __shfl_xor(ssq, 1);
        ssq += __shfl_xor(ssq, 2);
        ssq += __shfl_xor(ssq, 4);
        if ((f0 & 31) == 0) a.ssq[(size_t)(f0 >> 5) * a.Tp + t] = ssq;
    }
}

// state after the last committed pair <- state of phase row `row` (both layers are laid out back to back)
struct StateKeepArgs { float* state0; float* state1; int row, h; };
static __global__ __launch_bounds__(256) void k_state_keep(StateKeepArgs a) {
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= 2 * a.h) return;
    a.state0[(size_t)FV_MAX_TREE * 2 * a.h + idx] = a.state0[(size_t)a.row * 2 * a.h + idx];
    a.state1[(size_t)FV_MAX_TREE * 2 * a.h + idx] = a.state1[(size_t)a.row * 2 * a.h + idx];
}

// ============================================================================ outputs of a pass
// predicted feature rows: the block's residual stream after its MLP, fp32 [256 + KMAX][h] by output row id
struct DraftOutArgs { const float* x; float* fout; int r0, n, Tp, h; };
static __global__ __launch_bounds__(256) void k_draft_out(DraftOutArgs a) {
    const int t = blockIdx.x;
    if (t >= a.n) return;
    for (int f = threadIdx.x; f < a.h; f += 256)
        a.fout[(size_t)(a.r0 + t) * a.h + f] = a.x[((size_t)(f >> 2) * a.Tp + t) * 4 + (f & 3)];
}

// Top-m of one row of logits: descending value, lower token id first among equals (a total order, so
// the result is unique).  One workgroup of 1024 threads per row; a thread keeps 32 values in registers
// (vocabulary <= 32768).  The second best of every wavefront's 64 per-thread bests gives 32 values that
// reach the smallest of these sixteen, so that one is a threshold that at least 32 values reach: the
// values that reach it (usually about a hundred) are collected in LDS and ranked by counting.  If there
// are more than 256 of them (many equal logits), the list is instead drawn one winner per round.
// A row that holds a NaN or an infinity has no order: its list is filled with -1 and *bad is set.
struct TopmArgs {
    const float* logits;   // [n][Vpad] (row t of this pass)
    int32_t* top_tok;      // [256 + KMAX][FV_DRAFT_MMAX] by output row id
    float* top_val;
    int32_t* bad;          // set to 1 if some row is non-finite
    int r0, n, V, Vpad, m;
};

#define FV_TOPM_THREADS 1024
#define FV_TOPM_FAST 256   // candidates the counting path holds

// (value, token id) as one 64-bit integer, larger = earlier in the list; v is finite and not -0.  0 = no value.
__device__ __forceinline__ unsigned long long topm_key(float v, int i) {
    uint32_t u = __float_as_uint(v);
    u ^= (u >> 31) ? 0xFFFFFFFFu : 0x80000000u;
    return ((unsigned long long)u << 32) | (uint32_t)(0x7FFFFFFF - i);
}
__device__ __forceinline__ float topm_key_value(unsigned long long key) {
    uint32_t u = (uint32_t)(key >> 32);
    u ^= (u >> 31) ? 0x80000000u : 0xFFFFFFFFu;
    return __uint_as_float(u);
}
__device__ __forceinline__ int topm_key_token(unsigned long long key) { return 0x7FFFFFFF - (int)(uint32_t)key; }
__device__ __forceinline__ unsigned long long topm_wave_max(unsigned long long k) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const unsigned long long o = ((unsigned long long)(uint32_t)__shfl_xor((int)(k >> 32), off) << 32) | (uint32_t)__shfl_xor((int)(uint32_t)k, off);
        k = o > k ? o : k;
    }
    return k;
}

static __global__ __launch_bounds__(FV_TOPM_THREADS) void k_topm(TopmArgs a) {
    __shared__ unsigned long long wave_key[16];
    __shared__ unsigned long long cand[FV_TOPM_FAST];
    __shared__ int rank_of[FV_TOPM_FAST];
    __shared__ int n_cand, any_bad;
    const int t = blockIdx.x, tid = threadIdx.x, wave = tid >> 6;
    if (t >= a.n) return;
    const float* row = a.logits + (size_t)t * a.Vpad;
    if (tid == 0) { n_cand = 0; any_bad = 0; }
    if (tid < FV_TOPM_FAST) rank_of[tid] = 0;
    float x[32];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        const int v = (tid + FV_TOPM_THREADS * k) * 4;
        const float4 q = (v < a.V) ? *(const float4*)(row + v) : make_float4(0.f, 0.f, 0.f, 0.f);   // Vpad is a multiple of 32
        x[4 * k] = q.x + 0.f; x[4 * k + 1] = q.y + 0.f; x[4 * k + 2] = q.z + 0.f; x[4 * k + 3] = q.w + 0.f;   // -0 -> +0: equal values, one key
    }
    auto token_of = [&](int e) { return (tid + FV_TOPM_THREADS * (e >> 2)) * 4 + (e & 3); };   // ascending in e
    bool bad = false;
    float bv = -INFINITY;
    int bi = -1;
#pragma unroll
    for (int e = 0; e < 32; ++e)
        if (token_of(e) < a.V) {
            bad = bad || !(__builtin_fabsf(x[e]) < INFINITY);
            if (x[e] > bv) { bv = x[e]; bi = token_of(e); }   // the first of equal values stays
        }
    // the wavefront's best and second best of its 64 thread bests
    const unsigned long long my_key = (bi >= 0 && !bad) ? topm_key(bv, bi) : 0ull;
    const unsigned long long w1 = topm_wave_max(my_key);
    const unsigned long long w2 = topm_wave_max(my_key == w1 ? 0ull : my_key);   // keys of real values are distinct
    if ((tid & 63) == 0) wave_key[wave] = w2;
    if (__any(bad) && (tid & 63) == 0) any_bad = 1;   // written before the barrier, read after it (only ever set to 1)
    __syncthreads();
    int32_t* out_t = a.top_tok + (size_t)(a.r0 + t) * FV_DRAFT_MMAX;
    float* out_v = a.top_val + (size_t)(a.r0 + t) * FV_DRAFT_MMAX;
    if (tid < FV_DRAFT_MMAX) { out_t[tid] = -1; out_v[tid] = 0.f; }   // fewer than m tokens, or a non-finite row
    if (any_bad) {
        if (tid == 0) *a.bad = 1;
        return;
    }
    unsigned long long thr = wave_key[0];
#pragma unroll
    for (int w = 1; w < 16; ++w) thr = wave_key[w] < thr ? wave_key[w] : thr;   // 0 if some wavefront has fewer than two values: everything is a candidate
    const float tv = topm_key_value(thr);
    const int ti = topm_key_token(thr);
#pragma unroll
    for (int e = 0; e < 32; ++e) {
        const int i = token_of(e);
        const bool hit = i < a.V && (thr == 0ull || x[e] > tv || (x[e] == tv && i <= ti));
        if (hit) {
            const int pos = atomicAdd(&n_cand, 1);
            if (pos < FV_TOPM_FAST) cand[pos] = topm_key(x[e], i);
        }
    }
    __syncthreads();
    const int C = n_cand;
    if (C <= FV_TOPM_FAST) {
        // rank by counting: candidate c = tid % 256, a quarter of the comparisons per thread
        const int c = tid & (FV_TOPM_FAST - 1), part = tid >> 8;
        if (c < C) {
            const unsigned long long key = cand[c];
            int ahead = 0;
            for (int j = part; j < C; j += 4) ahead += cand[j] > key ? 1 : 0;
            if (ahead) atomicAdd(&rank_of[c], ahead);
        }
        __syncthreads();
        if (tid < C) {
            const int r = rank_of[tid];
            if (r < a.m && r < FV_DRAFT_MMAX) { out_t[r] = topm_key_token(cand[tid]); out_v[r] = topm_key_value(cand[tid]); }
        }
        return;
    }
    // many values reach the threshold (equal logits): one winner per round, each thread offering its best value
    // that comes after the last winner
    unsigned long long last = ~0ull;
    const int rounds = a.m < FV_DRAFT_MMAX ? a.m : FV_DRAFT_MMAX;
    for (int round = 0; round < rounds; ++round) {
        unsigned long long offer = 0ull;
#pragma unroll
        for (int e = 0; e < 32; ++e) {
            const int i = token_of(e);
            const unsigned long long k = i < a.V ? topm_key(x[e], i) : 0ull;
            offer = (k < last && k > offer) ? k : offer;
        }
        const unsigned long long w = topm_wave_max(offer);
        __syncthreads();   // the previous round's wave_key has been read by everyone
        if ((tid & 63) == 0) wave_key[wave] = w;
        __syncthreads();
        unsigned long long win = wave_key[0];
#pragma unroll
        for (int q = 1; q < 16; ++q) win = wave_key[q] > win ? wave_key[q] : win;
        if (win == 0ull) break;   // fewer than m tokens
        if (tid == 0) { out_t[round] = topm_key_token(win); out_v[round] = topm_key_value(win); }
        last = win;
    }
}

// tokens of the tree nodes a pass generates: node_tok[i] = top list of its generating row at its rank
struct ExpandArgs { DraftTables tab; const int32_t* top_tok; int32_t* node_tok; int e0, n; };
static __global__ __launch_bounds__(256) void k_draft_expand(ExpandArgs a) {
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j >= a.n) return;
    const int i = a.tab.exp_list[a.e0 + j];
    a.node_tok[i] = a.top_tok[(size_t)a.tab.node_gen[i] * FV_DRAFT_MMAX + a.tab.node_rank[i]];
}

// History of the last k-1 committed rows' outputs (predicted feature, top list), kept across phases in
// output rows 256 .. 256+k-2.  With C = [history, chain rows 0..n_prev-1 of the phase that ends], the new
// history is C[n_prev .. n_prev+k-2].  A new entry j only reads entries above j, so one workgroup moves
// them in ascending order.
struct HistArgs { float* fout; int32_t* top_tok; float* top_val; int n_prev, k, h; };
static __global__ __launch_bounds__(256) void k_draft_hist(HistArgs a) {
    for (int j = 0; j < a.k - 1; ++j) {
        const int c = a.n_prev + j;
        const int src = (c < a.k - 1) ? FV_MAX_TREE + c : c - (a.k - 1);
        const int dst = FV_MAX_TREE + j;
        for (int f = threadIdx.x; f < a.h; f += 256) a.fout[(size_t)dst * a.h + f] = a.fout[(size_t)src * a.h + f];
        if (threadIdx.x < FV_DRAFT_MMAX) {
            a.top_tok[dst * FV_DRAFT_MMAX + threadIdx.x] = a.top_tok[src * FV_DRAFT_MMAX + threadIdx.x];
            a.top_val[dst * FV_DRAFT_MMAX + threadIdx.x] = a.top_val[src * FV_DRAFT_MMAX + threadIdx.x];
        }
        __syncthreads();
    }
}

// plain fill (pad columns of activation buffers after a change of the row padding)
static __global__ __launch_bounds__(256) void k_draft_fill(uint32_t* p, uint32_t v, size_t n) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) p[i] = v;
}
