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
    FV_E_SCRATCH_LIMIT = -11  /* fv_verify_tree_noalloc: n_nodes > FV_NOALLOC_MAX_NODES, or the shape needs more
                                 scratch than the library's static device array holds */
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

#ifdef __cplusplus
}
#endif
#endif /* FALCON_VERIFY_H */
