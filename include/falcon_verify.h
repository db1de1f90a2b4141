/*
 * falcon_verify -- tree-verification step of Falcon's speculative decoding loop,
 * hand-written HIP for gfx950 (MI355X), behind a plain C ABI.
 *
 * The operation (paper, section "Custom-Designed Decoding Tree"; Appendix "Tree
 * Structure"; Experiments, "Models and Tasks"): the drafted tokens form a tree whose
 * nodes each stand for the candidate sequence spelled by their root path.  The target
 * LLM checks all candidates in ONE forward pass in which a node attends only to the
 * committed prefix and to its own ancestors (tree attention, SpecInfer-style
 * verification).  In the greedy setting (temperature 0, batch 1) a child is accepted iff
 * its parent is accepted and its token is the target's argmax at the parent; the longest
 * accepted path is kept together with the K/V computed for it, and the target's argmax at
 * the end of that path is the bonus token that becomes the next root.  The result is
 * token-for-token what plain greedy decoding would produce (the speed-up is lossless).
 *
 * Conventions
 *   - Node 0 is the root: the token the target produced last, not yet in the KV cache.
 *     It is always accepted.  Every other node holds exactly one draft token.
 *     parent[0] = -1, 0 <= parent[i] < i, depth[i] = depth[parent[i]] + 1.
 *   - L = number of tokens whose K/V are committed.  Node i sits at position L + depth[i].
 *   - accepted_len a = number of accepted DRAFT nodes (0 .. max depth); the step emits
 *     a + 1 tokens: accepted_tokens[0..a) then next_token.  Afterwards L += a + 1.
 *   - Ties: argmax takes the lowest token id; among accepted nodes of equal depth the
 *     lowest node index wins.
 *
 * Memory and ownership
 *   - All `const void*` / `int32_t*` arguments named host_* or documented "host" are
 *     host pointers owned by the caller; the library copies what it needs before it
 *     returns and never frees caller memory.
 *   - The device arena is ONE device allocation made by the caller (for instance a
 *     torch uint8 tensor) of at least fv_workspace_bytes() bytes, 256-byte aligned, that
 *     must outlive the context.  The library allocates no device memory itself.
 *   - `hip_stream` is a hipStream_t (or NULL for the default stream) on which all work of
 *     the context is enqueued.  Every call is synchronous on return: outputs are valid.
 *   - One context must not be used from two threads at once.
 *
 * Errors: every int-returning call gives FV_OK (0) or a negative fv_status.  Argument
 * and tree validation happens on the host before anything is launched; a rejected call
 * changes no state and writes no output.
 */
#ifndef FALCON_VERIFY_H
#define FALCON_VERIFY_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum fv_status {
    FV_OK = 0,
    FV_E_BAD_ARG = -1,        /* null pointer, unsupported shape, arena too small or misaligned */
    FV_E_TREE_ORDER = -2,     /* parent[0] != -1, or parent[i] outside [0, i) */
    FV_E_TREE_DEPTH = -3,     /* depth[i] != depth[parent[i]] + 1 (or depth[0] != 0) */
    FV_E_TOKEN_RANGE = -4,    /* a token id outside [0, vocab) */
    FV_E_TREE_TOO_BIG = -5,   /* n_nodes > max_tree */
    FV_E_CACHE_FULL = -6,     /* L + n_nodes > max_seq */
    FV_E_ROOT_MISMATCH = -7,  /* tree_tokens[0] is not the pending root token */
    FV_E_NO_PREFILL = -8,     /* verify_tree / rollback before prefill, or weights not set */
    FV_E_HIP = -9,            /* a HIP runtime call failed (no usable GPU, launch error) */
    FV_E_NONFINITE = -10,     /* the logits of some node hold a NaN or an infinity: there is no greedy choice;
                                 the committed length and the pending root are left as they were */
    FV_E_SCRATCH_LIMIT = -11, /* fv_verify_tree_noalloc: n_nodes > FV_NOALLOC_MAX_NODES, or the shape needs more
                                 scratch than the library's static device array holds */
    FV_E_EXCHANGE_TIMEOUT = -12 /* a GEMM workgroup waited about a third of a second for another workgroup's partial
                                 sums and gave up (a device so oversubscribed that the workgroups of one launch do
                                 not run together, or a device fault).  The step's results are invalid, every kernel
                                 still ran to its end, and the context (or drafter) returns this from every later
                                 step: destroy it. */
} fv_status;

enum { FV_F32 = 0, FV_BF16 = 1 };

/* Llama-style decoder shape (the model families of the paper's experiments): RMSNorm,
 * rotate-half rotary positions, grouped KV heads, SwiGLU FFN, no biases, untied head.
 * Supported: head_dim in {64, 128}; hidden, n_q_heads*head_dim multiples of 64;
 * ffn a multiple of 16; n_q_heads a multiple of n_kv_heads; 1 <= max_tree <= 256. */
typedef struct fv_cfg {
    int32_t n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn, vocab;
    int32_t dtype;     /* FV_F32: fp32 weights, activations and cache.
                          FV_BF16: bf16 weights, GEMM inputs and cache; fp32 accumulation,
                          residual stream, softmax and logits. */
    int32_t max_seq;   /* cache capacity in tokens (prefix + tree must fit) */
    int32_t max_tree;  /* largest n_nodes accepted by fv_verify_tree */
    float rope_base;   /* rotary base (10000 for the models in question) */
    float rms_eps;     /* epsilon inside the RMSNorm square root */
} fv_cfg;

/* Host pointers to the weights.  Matrices are row-major [out_features, in_features] in
 * cfg.dtype (fp32, or bf16 as raw 16-bit patterns); gains are fp32 vectors of `hidden`.
 * Per-layer members point to arrays of n_layers pointers. */
typedef struct fv_host_weights {
    const void* embed;            /* [vocab, hidden] */
    const void* lm_head;          /* [vocab, hidden] */
    const float* g_final;         /* [hidden] */
    const void* const* wq;        /* [n_q_heads*head_dim, hidden] */
    const void* const* wk;        /* [n_kv_heads*head_dim, hidden] */
    const void* const* wv;        /* [n_kv_heads*head_dim, hidden] */
    const void* const* wo;        /* [hidden, n_q_heads*head_dim] */
    const void* const* wg;        /* [ffn, hidden]  (gate) */
    const void* const* wu;        /* [ffn, hidden]  (up) */
    const void* const* wd;        /* [hidden, ffn]  (down) */
    const float* const* g_attn;   /* [hidden]  gain of the pre-attention norm */
    const float* const* g_mlp;    /* [hidden]  gain of the pre-FFN norm */
} fv_host_weights;

typedef struct fv_ctx fv_ctx;

/* Human-readable name of a status code (static string). */
const char* fv_status_str(int status);

/* Bytes of device arena a context of this shape needs.  Pure host arithmetic. */
int fv_workspace_bytes(const fv_cfg* cfg, size_t* out_bytes);

/* Host-only check of a tree against the rules above; exactly what fv_verify_tree runs
 * first.  `pending_root` is the token the root must carry, `cur_len` the committed
 * length L.  All pointers are host pointers.  No GPU needed. */
int fv_validate_tree(const fv_cfg* cfg, const int32_t* tree_tokens, const int32_t* parent_idx,
                     const int32_t* depth, int32_t n_nodes, int32_t pending_root, int32_t cur_len);

/* Create a context over a caller-owned device arena (device pointer) and stream.
 * Zero-fills the arena.  *out receives the context (host object, free with fv_destroy). */
int fv_create(const fv_cfg* cfg, void* dev_arena, size_t arena_bytes, void* hip_stream, fv_ctx** out);
void fv_destroy(fv_ctx* ctx);

/* Copy the weights to the device, re-tiled into the streaming layout of the skinny
 * GEMMs (each wavefront reads its weight tiles as fully contiguous 1 KiB lines).
 * The host arrays may be released afterwards. */
int fv_init_weights(fv_ctx* ctx, const fv_host_weights* host_weights);

/* Run a prompt of n >= 1 host tokens, fill cache slots 0..n-1, and return the target's
 * greedy next token in *next_token (host).  Resets the context state: L = n, pending
 * root = *next_token.  The prompt goes through the same kernels as verification, in
 * chain-shaped chunks of at most max_tree tokens. */
int fv_prefill(fv_ctx* ctx, const int32_t* host_tokens, int32_t n, int32_t* next_token);

/* One tree-verification step (the operation described at the top).  Inputs are host
 * arrays of n_nodes int32.  Outputs (host): *accepted_len = a; accepted_tokens[0..a)
 * (capacity >= the tree's maximum depth); *next_token.  On success the K/V of the
 * accepted path are compacted into cache slots L..L+a, L becomes L + a + 1 and the
 * pending root becomes *next_token. */
int fv_verify_tree(fv_ctx* ctx, const int32_t* tree_tokens, const int32_t* parent_idx,
                   const int32_t* depth, int32_t n_nodes,
                   int32_t* accepted_len, int32_t* accepted_tokens, int32_t* next_token);

/* One NON-greedy verification step: multi-step speculative sampling over the tree (Appendix "Tree
 * Structure": in a non-greedy setting a node's children are sampled instead of being the top-m
 * tokens; section "Custom-Designed Decoding Tree": the LLM verifies the tree in the SpecInfer manner).
 * The forward pass, K/V compaction, state update and read-back are those of fv_verify_tree; only the
 * acceptance rule differs.  With p = softmax(logits[node] / temperature) at the current node (the root
 * first), its children are tried in index order: child c with token x is accepted with probability
 * min(1, p[x] / q[x]) -- the test is u_accept[c] * q[x] <= p[x] -- and becomes the current node; on
 * rejection p becomes the normalised positive part of p - q.  When no child is accepted (or there is
 * none) next_token is drawn from what is left of p: the first token id v with cumsum(p)[v] >
 * u_sample[node].  Every emitted token is then distributed as the target's own sampling.
 *   temperature      > 0 (host value)
 *   dev_draft_probs  DEVICE pointer, fp32 row-major [n_nodes][vocab]: row i is the distribution the
 *                    drafter drew node i's children from (rows of leaves are not read); owned by the
 *                    caller, only read.  NULL: every child is its own point-mass proposal (q[x] = 1),
 *                    the right rule for deterministic (top-m) children: accept with probability p[x],
 *                    else strike x from p.
 *   u_accept, u_sample   HOST arrays of n_nodes doubles in [0, 1], drawn by the caller (the library
 *                    draws no random numbers): u_accept[c] decides node c, u_sample[i] the draw at node i.
 * The decisions are taken in fp64 from the fp32 logits.  Errors as fv_verify_tree, plus FV_E_BAD_ARG for
 * a bad temperature or a uniform outside [0, 1]. */
int fv_verify_tree_sampled(fv_ctx* ctx, const int32_t* tree_tokens, const int32_t* parent_idx,
                           const int32_t* depth, int32_t n_nodes,
                           float temperature, const float* dev_draft_probs,
                           const double* u_accept, const double* u_sample,
                           int32_t* accepted_len, int32_t* accepted_tokens, int32_t* next_token);

/* For callers that cannot allocate (code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc inside the step): fv_verify_tree with every scratch buffer of the step's
 * kernels (stream-K partial tiles and tickets, attention key-split partials and tickets) taken from
 * a static device array of 32 MiB inside the library instead of the arena's.  It calls no hipMalloc,
 * hipFree or other allocating routine.  Same arguments, outputs, errors and state changes as
 * fv_verify_tree, and bitwise the same results.  Limits: n_nodes <= FV_NOALLOC_MAX_NODES and a
 * model shape whose scratch fits the array (all shapes with at most 56 query heads of 128 and 256
 * GEMM workgroups do), else FV_E_SCRATCH_LIMIT and nothing is changed.  Every GPU the library has
 * created a context on holds its own copy of the array until the process ends; all contexts on one
 * GPU share it, so calls that overlap on one GPU (two streams, two threads) race.  The array keeps
 * the last call's contents; what must start at zero is cleared by a small kernel at each call. */
#define FV_NOALLOC_MAX_NODES 64
int fv_verify_tree_noalloc(fv_ctx* ctx, const int32_t* tree_tokens, const int32_t* parent_idx,
                           const int32_t* depth, int32_t n_nodes,
                           int32_t* accepted_len, int32_t* accepted_tokens, int32_t* next_token);

/* Step-invariant rows (paper, Abstract and section "Custom-Designed Decoding Tree": the output of
 * drafting plus verification is exactly the target's own greedy output).  With this on, the logits,
 * the K/V rows and the features of a node are bitwise the same whether the node is verified alone
 * (a one-node tree per step, i.e. plain decoding) or as one node of any tree of up to 64 nodes and
 * depth up to 32, so a decoding loop built on fv_verify_tree emits bit for bit what one-token steps
 * emit, top-2 near-ties included.  Off (the default), a node's attention sums are grouped by the
 * step's row count and by the cache slots its ancestors happen to occupy; rows then agree to
 * rounding level only (the 2e-2 parity bar holds either way) and a near-tie can tip.  It applies to
 * fv_verify_tree, fv_verify_tree_noalloc and fv_verify_tree_sampled; steps with more than 64 nodes
 * or deeper nodes, and fv_prefill, compute the same thing in the default form.  Costs attention
 * time (the last 33..64 positions of every node are summed per node in position order instead of
 * through shared matrix tiles); fv_verify_tree_noalloc then also needs the step's far-key parts to
 * fit its scratch (prefixes up to about 1300 tokens), else FV_E_SCRATCH_LIMIT.
 * enabled: 0 or 1.  May be changed between steps. */
int fv_set_step_invariant(fv_ctx* ctx, int32_t enabled);

/* Reset the committed length and pending root (0 <= new_len <= current capacity use is
 * the caller's responsibility: slots below new_len must hold valid K/V).  Used to replay
 * the same step and to resume. */
int fv_rollback(fv_ctx* ctx, int32_t new_len, int32_t pending_root);

/* Current committed length L and pending root token. */
int fv_get_state(fv_ctx* ctx, int32_t* cur_len, int32_t* pending_root);

/* ---- read-back of the last fv_verify_tree / fv_prefill chunk (host output buffers) ---- */

/* Ancestor sets as computed on the device: n_nodes x 4 little-endian 64-bit words,
 * bit j of node i's set in word j/64, bit j%64. */
int fv_get_tree_mask(fv_ctx* ctx, uint64_t* out_words, int32_t n_nodes);
/* Logits of every node, row-major [n_nodes, vocab] fp32. */
int fv_get_logits(fv_ctx* ctx, float* out, int32_t n_nodes);
/* Per-node argmax token ids. */
int fv_get_argmax(fv_ctx* ctx, int32_t* out, int32_t n_nodes);
/* Compaction moves of the last verify: src_slot[j] = tree index of path node j,
 * dst_slot[j] = cache slot it was copied to; *count = a + 1.  Capacity >= max_tree. */
int fv_get_kv_moves(fv_ctx* ctx, int32_t* src_slot, int32_t* dst_slot, int32_t* count);
/* Features of the accepted path of the last fv_verify_tree, for the next drafting round (section
 * "Custom-Designed Decoding Tree": the accepted tokens are recorded together with their
 * features; section "Framework": the drafter consumes the LLM's last-layer features, shifted by
 * one against the tokens).  Row j, j = 0..accepted_len, is the LM head's input of path node j --
 * the last layer's output after the final RMSNorm (the paper does not say before or after that
 * norm; after is what the shared LM head consumes) -- as fp32, row-major [n_rows, hidden].
 * out: host buffer; n_rows in 1..accepted_len+1, else FV_E_BAD_ARG; nothing is changed. */
int fv_get_features(fv_ctx* ctx, float* out, int32_t n_rows);
/* K (after rotation) and V of cache slots [slot0, slot0+n) of one layer, as fp32
 * [n, n_kv_heads, head_dim] each, in logical order. */
int fv_read_kv(fv_ctx* ctx, int32_t layer, int32_t slot0, int32_t n, float* k_out, float* v_out);

/* Intermediate activations of the LAST layer the last step ran, for bring-up and parity
 * tests: out is row-major [n_nodes, n_features] fp32.  which: FV_ACT_X residual stream
 * after the layer (hidden features); FV_ACT_XB the next GEMM input x * gain, before the
 * RMSNorm factor (hidden); FV_ACT_Q rotated queries (n_q_heads*head_dim); FV_ACT_ATTN
 * attention output (n_q_heads*head_dim); FV_ACT_FFN silu(gate)*up (ffn). */
enum { FV_ACT_X = 0, FV_ACT_XB = 1, FV_ACT_Q = 2, FV_ACT_ATTN = 3, FV_ACT_FFN = 4 };
int fv_debug_read_activation(fv_ctx* ctx, int32_t which, int32_t n_nodes, float* out);

/* ---- measurement ---- */

/* Context for the roofline figures: the rate in GB/s (1e9 bytes) at which a plain streaming-read kernel of
 * the library (one workgroup per compute unit, contiguous 16-byte loads) reads the context's tiled weights
 * (the first 4 GiB of them at most) `passes` times (1..64) on the context's stream, after one untimed pass.
 * Writes nothing the step uses.  *gbytes_per_s: host output. */
int fv_stream_read(fv_ctx* ctx, int32_t passes, float* gbytes_per_s);

/* When enabled, each subsequent step brackets its kernels with HIP events on the
 * context's stream and accumulates per-phase device time.  Off by default (the events
 * cost launch gaps). */
int fv_set_profiling(fv_ctx* ctx, int32_t enabled);
/* phases: the weight-streaming GEMM kernels; the separate reduction launches of steps of more than
 * 64 rows; tree attention kernels; everything else (ingest, embedding, argmax, path scan, compaction) */
enum { FV_PH_GEMM = 0, FV_PH_FIXUP = 1, FV_PH_ATTN = 2, FV_PH_OTHER = 3, FV_PH_COUNT = 4 };
/* Accumulated milliseconds and launch counts per phase since the last reset; reading
 * resets them.  Arrays of FV_PH_COUNT. */
int fv_get_phase_times(fv_ctx* ctx, float* ms, int32_t* launches);
/* Device time in ms of the last step's kernels (first launch to last), measured with
 * HIP events on the context's stream.  Always available. */
int fv_last_step_ms(fv_ctx* ctx, float* ms);

/* ============================================================================================
 * Drafting phase: the SAR head of the paper (sections "Framework and Computational Process",
 * "Coupled Sequential Glancing Distillation", "Custom-Designed Decoding Tree"; Appendix "Tree
 * Structure").  The drafter is the target's embedding table, two LSTM layers that take the
 * concatenation [feature of position j ; embedding of token j+1] (width 2*hidden) down to hidden,
 * one decoder block of the target's geometry under the relaxed causal mask (a row sees its
 * predecessors in the tree and every row of its own block of k rows), and the target's LM head.
 * The row at position j predicts the feature of position j+k, so one pass over a block of k rows
 * yields the distributions of the next k tokens; node i of the static tree at depth d takes the
 * token of rank rank[i] (0 = most likely; ties: lower token id first) of the distribution of its
 * depth.  The paper fixes neither dimensions nor wiring; the choices made here are listed in the
 * design notes and implemented identically by the CPU oracle.
 *
 * State: the drafter keeps its own K/V cache and LSTM state over the committed pairs.  A phase is
 *   fv_draft_commit (the pairs the target fixed since the last phase: n = accepted + 1 after a
 *   verification step, the whole prompt after prefill), then at most one fv_draft_tree.
 * Limits: k <= FV_DRAFT_MAX_K; rank < FV_DRAFT_MAX_M; at most 256 rows per phase (rows of the
 *   commit's last piece + rows of all blocks); vocab <= 32768.
 * The drafter shares the target context's stream, embedding table and LM head: the target context
 * must outlive it and its weights must be set.  Calls are synchronous on return. */
#define FV_DRAFT_MAX_K 8
#define FV_DRAFT_MAX_M 32

typedef struct fv_drafter fv_drafter;

/* Host pointers; matrices row-major [out, in] in the target's dtype, biases and gains fp32.
 * LSTM gate rows are ordered input, forget, cell, output; layer 0 is [4h, 2h] / [4h, h], layer 1
 * [4h, h] / [4h, h]; one bias vector [4h] per layer. */
typedef struct fv_drafter_host_weights {
    const void* lstm_w_ih[2];
    const void* lstm_w_hh[2];
    const float* lstm_b[2];
    const void *wq, *wk, *wv, *wo, *wg, *wu, *wd;   /* the decoder block, shapes as in fv_host_weights */
    const float *g_attn, *g_mlp;
} fv_drafter_host_weights;

/* Bytes of device arena a drafter for a target of this shape needs.  Pure host arithmetic. */
int fv_drafter_workspace_bytes(const fv_cfg* target_cfg, size_t* out_bytes);

/* Create a drafter over a caller-owned device arena (256-byte aligned, zero-filled here). */
int fv_drafter_create(fv_ctx* target, int32_t k, void* dev_arena, size_t arena_bytes, fv_drafter** out);
void fv_drafter_destroy(fv_drafter* d);
int fv_drafter_init_weights(fv_drafter* d, const fv_drafter_host_weights* host_weights);

/* Forget all committed pairs (zero LSTM state, empty cache). */
int fv_draft_reset(fv_drafter* d);

/* Take in n >= 1 pairs the target has fixed: host_tokens[i] = token of position L+i+1,
 * dev_features = DEVICE pointer to n rows of `hidden` fp32 (row i = the target's feature of
 * position L+i, i.e. its LM-head input; for instance what fv_features_device_ptr gives after a
 * verification step).  Rows are processed in sequence order under a causal mask; their K/V and
 * the LSTM state are kept, L += n.  Opens a new phase. */
int fv_draft_commit(fv_drafter* d, const int32_t* host_tokens, const float* dev_features, int32_t n);

/* Fill a static tree with draft tokens.  parent / depth as for fv_verify_tree (node 0 = root =
 * the token of the last committed pair, root_token); rank[i] = rank of node i among the
 * candidates of its place.  tokens_out (host, n_nodes) receives the tree's tokens, ready for
 * fv_verify_tree.  ceil(max depth / k) - 1 passes run (the first k levels come from the rows
 * of the commit).  Needs at least k committed pairs and an open phase. */
int fv_draft_tree(fv_drafter* d, const int32_t* parent_idx, const int32_t* depth, const int32_t* rank, int32_t n_nodes,
                  int32_t root_token, int32_t* tokens_out);

/* Read-back (tests): committed pairs, rows of the current phase, rows of its commit. */
int fv_draft_get_state(fv_drafter* d, int32_t* committed, int32_t* phase_rows, int32_t* chain_rows);
enum { FV_DRAFT_FEATURES = 0, FV_DRAFT_LOGITS = 1 };
/* Predicted features [n, hidden] or logits [n, vocab] of phase rows row0.. (host, fp32). */
int fv_draft_get_rows(fv_drafter* d, int32_t what, int32_t row0, int32_t n, float* out);
/* Top lists [n, FV_DRAFT_MAX_M] of phase rows row0.. (host). */
int fv_draft_get_top(fv_drafter* d, int32_t row0, int32_t n, int32_t* tokens_out);
/* K and V of the drafter's cache slots (layout as fv_read_kv). */
int fv_draft_read_kv(fv_drafter* d, int32_t slot0, int32_t n, float* k_out, float* v_out);
/* Device time of the last fv_draft_commit / fv_draft_tree in milliseconds. */
int fv_draft_last_ms(fv_drafter* d, float* ms);
/* DEVICE address of the feature rows the last verification step exported (what fv_get_features copies). */
int fv_features_device_ptr(fv_ctx* ctx, const float** dev_rows);

#ifdef __cplusplus
}
#endif
#endif /* FALCON_VERIFY_H */
