/*
 * adore.h - C ABI of the ADORE decode-step library for MI355X (gfx950).
 *
 * One context holds the state of one decode job of B sequences: per layer a
 * fixed-size, slot-addressed K/V cache of K rows per (sequence, head), the
 * per-token keep probabilities sigma_i, and the controller's GRU state.
 * One decode step = the four stages of the paper's method (arXiv 2407.02328):
 *
 *   attend    single-query attention over the occupied slots, the current
 *             token's k, v included                       (Sec. 2.1, Eq. 1 and
 *                                                          the "target" equation)
 *   schedule  controller score of the arriving token       (Sec. 2.2, Eq. 2;
 *             App. "Implementation Details", controller module),
 *             release of the lowest-scored rows            (Sec. 2.2, third
 *                                                          design strategy),
 *             choice of the top-R released tokens          (Sec. 2.3)
 *   rebuild   K/V of the chosen tokens re-projected from their hidden states
 *             with W_k / W_v and written into the freed slots (Sec. 2.3)
 *
 * Symbols: L layers, B sequences, H heads, d head_dim, D hidden size, K cache
 * slots per (sequence, head), R rebuild budget per step and sequence,
 * m = K - R - 1 persistent rows, d' controller hidden size, n = 0-based
 * position of the current token, S prompt length.
 *
 * Conventions
 *   - Every pointer is a DEVICE pointer unless its comment says HOST.  The two
 *     structs below are read on the host.
 *   - All arrays are contiguous, row-major, last index fastest, bases 16-byte
 *     aligned.  "storage type" is adore_config.dtype (bf16 or fp32).
 *   - The caller owns all memory.  The library allocates no device memory; the
 *     workspace passed to adore_create holds all of its state.
 *   - attend / schedule / rebuild / decode_step only enqueue work on the
 *     context's stream and never synchronise it: outputs are valid once the
 *     caller has synchronised that stream.  Input buffers must stay unchanged
 *     until then.  Inputs may be produced by work enqueued on that stream before
 *     the call (see adore_set_input_order for the one exception a caller can
 *     ask for).
 *   - The return value is the only error channel.  Arguments and the order of
 *     calls are validated on the host before anything is enqueued: a call that
 *     returns E_INVALID, E_STATE, E_UNSUPPORTED or E_WORKSPACE has had no effect.
 *     E_HIP means the HIP runtime refused something in the middle of a call;
 *     part of the step may have been enqueued, and the context has to be
 *     restarted with adore_init_cache (or adore_set_state) before its next step.
 *   - A context is bound to one stream and is not thread-safe.  Contexts are
 *     independent of each other.
 *   - Ties between equal sigma are broken in favour of the lower position, so
 *     every selection has exactly one result.  A NaN sigma is treated as 0.
 */
#ifndef ADORE_H
#define ADORE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ADORE_ABI_VERSION 10

typedef struct adore_ctx adore_ctx; /* opaque */

enum { ADORE_F32 = 0, ADORE_BF16 = 1 };

/* When the controller's score of a token is taken (the two readings of Sec. 2.2):
 * STATIC:  sigma_i once, when token i arrives, with the position feature i * pos_scale (Eq. 2 as printed).
 * RESCORE: at every step n, sigma_i for every token i <= n from its stored GRU state z_i with the
 *          position feature (n - i) * pos_scale (the controller rates the cached tokens "for the current
 *          token", Sec. 2.2 and the caption of Fig. 2); both selections of the step use the new values,
 *          so a rebuilt token can be kept.  score_override must be NULL in every call, set_state is
 *          not available, and d' must be a multiple of 4. */
/* H2O:     the H2O(Rebuilt) baseline of Sec. 3.1 (baselines 6 and 7): no controller; the score of a token is the
 *          attention it has received so far, kept per head: score[b][h][i] = sum over the steps at which head h
 *          held a row of token i of the probability the step's query gave that row (fp32, added in step order; an
 *          evicted token keeps its score and collects again once rebuilt).  Every head releases on its own scores
 *          and has its own slot map.  The rebuild is per sequence (one row of the re-projection serves all heads):
 *          candidates are the tokens at least one head is missing, ranked by the fp32 sum of their scores over the
 *          heads (head 0 first), equal sums to the lower position; a head that still holds a chosen token keeps its
 *          row, the others put it into their lowest free slots in rank order.  (The paper gives the baseline two
 *          sentences; the rest is this reading.)  One layer per context, no rotary embedding, heads <= 255,
 *          max_positions <= about 7000 (the keys of a sequence live in 64 KB of LDS; fewer with a large R); x_n and the controller weights are not read (x_n may be NULL, the weight
 *          pointers must still be non-null); score_override of adore_init_cache is [B][H][S], the attention the
 *          prompt tokens collected during the prompt (NULL: zeros), and must be NULL in the step calls; the scores
 *          of get_state are [B][H][N_max]; no set_state, no adore_forward_step. */
enum { ADORE_SCORE_STATIC = 0, ADORE_SCORE_RESCORE = 1, ADORE_SCORE_H2O = 2 };

enum {
  ADORE_OK = 0,
  ADORE_E_INVALID = -1,     /* null pointer, bad shape or value */
  ADORE_E_STATE = -2,       /* call out of order, or step past max_positions */
  ADORE_E_UNSUPPORTED = -3, /* valid in principle, no kernel for it */
  ADORE_E_WORKSPACE = -4,   /* workspace too small or misaligned */
  ADORE_E_HIP = -5          /* a HIP runtime call failed */
};

typedef struct {
  int32_t layers, batch, heads, head_dim, hidden;     /* L, B, H, d, D */
  int32_t cache_slots, rebuild_budget, max_positions; /* K, R (0 <= R <= K-2), N_max */
  int32_t ctrl_hidden;                                /* d' */
  int32_t dtype;                                      /* ADORE_F32 | ADORE_BF16 */
  float pos_scale;                                    /* position feature of token i = (float)i * pos_scale */
  int32_t score_mode;                                 /* ADORE_SCORE_STATIC | ADORE_SCORE_RESCORE | ADORE_SCORE_H2O */
  float rope_base;                                    /* 0: off.  > 0: rotary position embedding (the one the paper's
                                                         backbones apply to q and k; the paper names it in its related
                                                         work on length extrapolation) on every key the library makes
                                                         from a hidden state, and on the queries of the rebuild forward:
                                                         the projection is rounded to the storage type, elements j and
                                                         j + d/2 of each head are turned by pos * rope_base^(-2j/d), and
                                                         the result is rounded again.  Keys and queries the caller
                                                         supplies (prompt_k, k_new, q) are taken as they are. */
} adore_config;

/* Device pointers, caller-owned, read-only, must outlive the context. */
typedef struct {
  const void *w_kv;      /* [L][2*H*d][D] storage type; rows 0..H*d-1 = W_k, the rest = W_v;
                            within each half, rows h*d..h*d+d-1 belong to head h */
  const void *gru_w_ih;  /* [3*d'][D]  storage type, gate order r, z, n */
  const void *gru_w_hh;  /* [3*d'][d'] storage type, gate order r, z, n */
  const float *gru_b_ih; /* [3*d'] */
  const float *gru_b_hh; /* [3*d'] */
  const float *pos_w;    /* [d']      position layer, 1 -> d' */
  const float *pos_b;    /* [d'] */
  const float *mlp_w1;   /* [d'][d']  interaction layer (tanh) */
  const float *mlp_b1;   /* [d'] */
  const float *out_w;    /* [d']      output layer (sigmoid) */
  const float *out_b;    /* [1] */
} adore_weights;

/* Bytes of device workspace adore_create needs for this configuration (0 if the
 * configuration is invalid).  HOST call, no GPU work. */
size_t adore_workspace_bytes(const adore_config *cfg);

/* Creates a context over `workspace` (device memory, 256-byte aligned, at least
 * adore_workspace_bytes(cfg) bytes, owned by the caller and kept alive until
 * adore_destroy).  `hip_stream` is a hipStream_t (NULL = the default stream).
 * cfg and weights are HOST structs and are copied.  The cache starts empty;
 * call adore_init_cache before the first step.
 * Errors: E_INVALID (null, R > K-2, sizes <= 0, or sizes beyond what 32-bit counts hold with a wide
 * margin: L > 4096, B*H > 2^20, H*d or D > 2^20, K > 2^20, N_max > 2^24), E_UNSUPPORTED (head_dim not in
 * {64,128}, K > 1024 unless K - R - 1 >= N_max, i.e. a cache that holds every
 * token and is the full attention of Eq. 1 ... see adore_strerror), E_WORKSPACE. */
int adore_create(const adore_config *cfg, const adore_weights *weights, void *workspace,
                 size_t workspace_bytes, void *hip_stream, adore_ctx **out);

/* Frees the host-side context.  Does not touch device memory. */
int adore_destroy(adore_ctx *ctx);

/* Loads a prompt of S >= 1 tokens (the paper's user input t_1..t_s, Sec. 2.1) by
 * applying the step rules once: the controller scores tokens 0..S-1 in order
 * (Eq. 2); the residents are token S-1 plus the best min(S,m)-1 older tokens,
 * placed from slot 0 in ascending position with the given K/V; the best
 * min(R, rest) of the remaining tokens are rebuilt from hidden_store into the
 * next slots by rank.
 *   prompt_k, prompt_v  [L][B][H][S][d]  storage type
 *   hidden_store        [L][B][N_max][D] storage type, rows < S valid
 *   ctrl_input          [B][S][D]        storage type (token embeddings x_i)
 *   score_override      [B][S] fp32 or NULL: if given, replaces the controller's sigma
 * hidden_store == NULL prepares the context for adore_forward_step instead: the best min(R, rest)
 * tokens are chosen and given their slots, but their K/V are computed by the first forward step.
 * Enqueues work; does not synchronise.  May be called again to restart.
 * Errors: E_INVALID (null, S < 1, S >= N_max), E_UNSUPPORTED (hidden_store == NULL and K > 8192 or
 * H2O scores: see adore_forward_step). */
int adore_init_cache(adore_ctx *ctx, const void *prompt_k, const void *prompt_v,
                     const void *hidden_store, const void *ctrl_input,
                     const float *score_override, int32_t S);

/* Stage 1 for one layer (Sec. 2.1): writes k_new, v_new into the slot reserved
 * for the current token and computes
 *   out[b][h][:] = sum_k softmax_k(q . Kc[k] / sqrt(d)) Vc[k]  over occupied slots.
 *   q, k_new, v_new  [B][H][d] storage type;  out [B][H][d] fp32.
 * Each layer must be attended exactly once per step, before adore_schedule.
 * Errors: E_INVALID, E_STATE (no init, layer already attended, step past N_max). */
int adore_attend(adore_ctx *ctx, int32_t layer, const void *q, const void *k_new,
                 const void *v_new, float *out);

/* Stages 2 and 3, once per step for all layers (uniform policy, Sec. 2.2):
 * sigma_n from the controller (Eq. 2) or from score_override; release of the
 * x = max(0, occupied - m) lowest-ranked rows of every (b,h), never the current
 * token; choice of the best min(R, pool) released tokens per sequence
 * (Sec. 2.3); assignment of rebuilt rank rho to the rho-th lowest free slot.
 *   x_n             [B][D] storage type (embedding of the current token)
 *   score_override  [B] fp32 or NULL
 *   slot_map        [B][H][K] i32 or NULL: position held by each slot after the
 *                   step, -1 = free
 *   released_pos    [B][H][R+1] i32 or NULL: released positions in ascending slot
 *                   order, -1 padded
 *   rebuilt_pos     [B][max(R,1)] i32 or NULL: chosen positions best first, -1 padded
 * Errors: E_INVALID, E_STATE (a layer not yet attended, schedule already done). */
int adore_schedule(adore_ctx *ctx, const void *x_n, const float *score_override,
                   int32_t *slot_map, int32_t *released_pos, int32_t *rebuilt_pos);

/* Stage 4 for one layer (Sec. 2.3): for each chosen token, one rounding to the
 * storage type of W_kv[layer] . hidden_store_layer[b][pos] (fp32 accumulation),
 * head slices scattered into the slots assigned by adore_schedule.
 *   hidden_store_layer  [B][N_max][D] storage type; rows of all positions <= n valid
 * Each layer must be rebuilt exactly once per step, after adore_schedule; the
 * step completes (n advances) when the last layer is rebuilt.
 * Errors: E_INVALID, E_STATE. */
int adore_rebuild(adore_ctx *ctx, int32_t layer, const void *hidden_store_layer);

/* The whole step for L == 1: attend(0); schedule; rebuild(0).
 *   q, k_new, v_new [B][H][d]; hidden_store [B][N_max][D]; x_n [B][D];
 *   score_override [B] or NULL; out [B][H][d] fp32; slot_map [B][H][K] or NULL.
 * Errors: as the three calls; E_INVALID if L != 1. */
int adore_decode_step(adore_ctx *ctx, const void *q, const void *k_new, const void *v_new,
                      const void *hidden_store, const void *x_n, const float *score_override,
                      float *out, int32_t *slot_map);

/* Rebuild forward through the layer stack (Sec. 2.3 in full: "the embeddings of the top-R released tokens
 * are concatenated with the current token" and go through every layer as R+1 query rows, whose
 * outputs are the next layer's inputs).  One call is one whole step for all L layers; it replaces
 * attend / schedule / rebuild, which need the caller to supply per-layer hidden states.
 * Rows of a sequence: the r tokens chosen by the previous step (or by adore_init_cache), by rank, then the
 * current token n.  Per layer l, with x the rows entering the layer (layer 0: their embeddings):
 *   q = round(W_q[l] x), [k; v] = round(W_kv[l] x)      k, v go to the rows' cache slots
 *   o[j] = softmax over the slots whose position is <= position(j) of q[j] . Kc / sqrt(d), times Vc
 *          (the paper prints no mask for these rows; a decoder's causal rule is used, so a rebuilt
 *           state equals the state the token had when all earlier tokens are present)
 *   x'   = round(x + W_o[l] round(o))                   a layer is attention + residual only: norms and
 *                                                        feed-forward belong to the backbone model
 * then the controller, the release and the choice of the next r tokens as in adore_schedule.
 *   fw->w_q   [L][H*d][D]  storage type, rows grouped by head like W_k
 *   fw->w_o   [L][D][H*d]  storage type
 *   embed     [B][N_max][D] storage type: token embeddings, rows of all positions <= n valid
 *   score_override, slot_map, released_pos, rebuilt_pos: as adore_schedule
 *   rows_out  [B][R+1][D] storage type: the last layer's rows; rank j at [b][j], the current token
 *             at [b][R]; rows of unused ranks are left untouched
 *   layer_rows [L][B][R+1][D] storage type or NULL: the rows leaving every layer (the hidden states of the
 *             rebuilt tokens and of the current one, layer by layer), laid out like rows_out; [L-1] equals rows_out
 * Requires a context initialised with hidden_store == NULL and K <= 8192.  bf16 storage with H*d and D
 * multiples of 128 runs the projections on the matrix cores, and with R + 1 <= 64 the attention too; any
 * other configuration (fp32 storage, other widths, more rows) takes plain kernels for that part, one wave
 * per output element: the same arithmetic in fp32, a reference path rather than a fast one.
 * Enqueues work; does not synchronise.
 * Errors: E_INVALID, E_STATE (not initialised for the forward, step past N_max). */
typedef struct {
  const void *w_q;
  const void *w_o;
} adore_forward_weights;
int adore_forward_step(adore_ctx *ctx, const adore_forward_weights *fw, const void *embed,
                       const float *score_override, void *rows_out, void *layer_rows, int32_t *slot_map,
                       int32_t *released_pos, int32_t *rebuilt_pos);

/* Snapshot / restore between steps.  Any pointer may be NULL (skipped).
 *   slot_pos [B][H][K] i32; scores [B][N_max] fp32; z [B][d'] fp32;
 *   cache_k, cache_v [L][B][H][K][d] storage type; step: HOST pointer, the
 *   position n of the next token.
 * get enqueues device-to-device copies (no synchronisation; *step is written at
 * once).  set copies, then SYNCHRONISES the stream to recount the occupied
 * slots; slot_pos must be given and must leave at least one free slot per (b,h).
 * Errors: E_INVALID, E_STATE (in the middle of a step). */
int adore_get_state(adore_ctx *ctx, int32_t *slot_pos, float *scores, float *z,
                    void *cache_k, void *cache_v, int32_t *step);
int adore_set_state(adore_ctx *ctx, const int32_t *slot_pos, const float *scores,
                    const float *z, const void *cache_k, const void *cache_v, int32_t step);

/* Input order.  The controller and the selections of a step run on a stream of the
 * context's own, next to the attention and the rebuild; they read x_n / embed and
 * score_override.  ordered != 0 (the default): they start behind everything that was
 * enqueued on the context's stream before the call, so those inputs may come from
 * kernels enqueued there, at the price of one more cross-stream event per step.
 * ordered == 0: the caller guarantees that x_n (embed) and score_override of a step
 * are complete in memory when the step's call is made (say, the token's embedding
 * was gathered before the stream was last synchronised); that event is dropped and
 * the side work of later steps may start early.  All other inputs are read on the
 * context's stream in either mode.  Outputs with ordered == 0: slot_map, released_pos
 * and rebuilt_pos of a step may then be written as soon as its call is made, ahead of
 * work queued on the context's stream; a caller whose earlier work on that stream
 * still reads the previous step's values gives each step buffers of its own (or
 * synchronises first).  `out` and rows_out are written on the context's stream.
 * The first step after adore_init_cache starts behind the init in either mode.
 * HOST call between steps.
 * Errors: E_INVALID, E_STATE (in the middle of a step). */
int adore_set_input_order(adore_ctx *ctx, int32_t ordered);

/* Per-kernel timing with HIP events on the context's stream (for benchmarks).
 * While enabled, every kernel launch is bracketed by two events.
 * adore_read_timing SYNCHRONISES the stream, adds up the elapsed milliseconds
 * per kernel since the last read into ms[ADORE_N_KERNELS] and the launch counts
 * into launches[ADORE_N_KERNELS] (both HOST arrays), and clears the record. */
enum {
  ADORE_KERNEL_ATTEND = 0,      /* insert + attention (partials when a row is split) */
  ADORE_KERNEL_ATTEND_COMBINE,  /* merge of the split partials; not launched for one split */
  ADORE_KERNEL_CTRL_INPUT,      /* GRU input projection */
  ADORE_KERNEL_CTRL_CELL,       /* GRU cell + MLP + sigmoid */
  ADORE_KERNEL_RELEASE,         /* per-(b,h) release select */
  ADORE_KERNEL_REBUILD_SELECT,  /* per-sequence top-R select + slot assignment */
  ADORE_KERNEL_REBUILD_GEMM,    /* re-projection + scatter */
  ADORE_KERNEL_RESCORE,         /* RESCORE mode: sigma of every token for the current step */
  ADORE_KERNEL_FWD_QKV,         /* rebuild forward: q, k, v projection of the rebuilt tokens' rows + scatter */
  ADORE_KERNEL_FWD_QKV_CUR,     /* rebuild forward: the same for the current tokens' rows (one per sequence) */
  ADORE_KERNEL_FWD_ATTEND,      /* rebuild forward: attention of the R+1 rows */
  ADORE_KERNEL_FWD_OPROJ,       /* rebuild forward: output projection + residual, rebuilt tokens' rows */
  ADORE_KERNEL_FWD_OPROJ_CUR,   /* rebuild forward: the same for the current tokens' rows */
  ADORE_KERNEL_ROPE,            /* rotary embedding of the rows a projection just wrote (rope_base > 0) */
  ADORE_KERNEL_H2O_RELEASE,     /* H2O mode: the step's attention added to the scores, then the per-head release */
  ADORE_KERNEL_H2O_CHOICE,      /* H2O mode: per-sequence choice of the tokens to rebuild on the sum over heads */
  ADORE_KERNEL_H2O_PLACE,       /* H2O mode: per head, the slots of the chosen tokens it is missing */
  ADORE_N_KERNELS
};
int adore_set_timing(adore_ctx *ctx, int32_t enable);
int adore_read_timing(adore_ctx *ctx, float *ms, int32_t *launches);
const char *adore_kernel_name(int32_t kernel);

/* Top-K attention over a whole sequence (Sec. 2.1: keeping the highest of a query's full weights is the ideal
 * sparsity; Sec. 2.2, first strategy, and App. "Implementation Details": the attention the backbone is fine-tuned
 * with, the weights outside the top K masked out).  Stateless: no context.  Causal, per row (= sequence x head):
 *   w[i][j] = q_i . k_j for j <= i;  query i keeps its top_k largest weights (all while i + 1 <= top_k; equal
 *   weights go to the lower j);  out_i = sum over the kept j of softmax_j(w[i][j] / sqrt(head_dim)) v_j.
 * q, k, v, out: DEVICE [rows][seq][head_dim] bf16, dense; out may not alias the inputs.  workspace: DEVICE,
 * 256-byte aligned, at least adore_topk_attention_workspace_bytes(rows, seq, head_dim) bytes (a transposed copy of
 * v; for seq > 2048 also the weights of the query blocks in flight, 512 * 16 * (seq + 36) * 4 bytes or so, which
 * shorter sequences keep on chip), caller-owned, free to reuse after the work enqueued here has run.  The call only enqueues work on
 * hip_stream (a hipStream_t, NULL = the default stream).  The selection is exact on the weights as the kernel
 * computes them (bf16 products accumulated in fp32); inputs must be finite.
 * Errors: E_INVALID (null, sizes <= 0, top_k < 1), E_UNSUPPORTED (head_dim not in {64,128}, seq > 32768,
 * rows > 65535), E_WORKSPACE, E_HIP.  adore_topk_attention_workspace_bytes is a HOST call and returns 0 for
 * sizes the entry point would not take. */
size_t adore_topk_attention_workspace_bytes(int32_t rows, int32_t seq, int32_t head_dim);
int adore_topk_attention(const void *q, const void *k, const void *v, void *out, void *workspace,
                         size_t workspace_bytes, int32_t rows, int32_t seq, int32_t head_dim, int32_t top_k,
                         void *hip_stream);

/* adore_topk_attention for callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid it): the same kernels and the same result, bit for bit, with the transposed copy of v
 * in a fixed array inside the library (ADORE_TOPK_STATIC_SCRATCH_BYTES of device memory on every GPU the library is
 * loaded on, held until the process ends) instead of a caller's workspace.  The call allocates and frees nothing.
 * Limits: seq <= 2048 and rows * head_dim * ceil(seq / 32) * 64 <= ADORE_TOPK_STATIC_SCRATCH_BYTES, else E_WORKSPACE
 * (e.g. 256 rows of 1024 tokens at head_dim 128).  All calls on one GPU share that array: calls whose work may
 * overlap on a GPU (different streams, different threads) race; calls on one stream are safe.  Nothing in the array
 * has to be cleared between calls (every call writes all of what it then reads).  The first call on a device looks
 * the array's address up (hipGetSymbolAddress), so make that call outside a graph capture.
 * Errors: as adore_topk_attention; E_WORKSPACE when the shape exceeds the array. */
#define ADORE_TOPK_STATIC_SCRATCH_BYTES (64u << 20)
int adore_topk_attention_static(const void *q, const void *k, const void *v, void *out, int32_t rows, int32_t seq,
                                int32_t head_dim, int32_t top_k, void *hip_stream);

const char *adore_strerror(int code);
/* Debug aid for callers and tests, not a step of the method (no passage of the paper): with ADORE_GUARD_WORDS=1
 * in the environment of the process, adore_workspace_bytes and adore_create lay the workspace out with 256 bytes of
 * a fixed pattern behind each of its regions (cache, slot maps, scores, lists, scratch).  No kernel has a reason to
 * touch them; a kernel that writes past the end of a region does.  adore_check_guards waits for the context's
 * streams and writes to *damaged (host) the number of 4-byte guard words that no longer hold the pattern: 0 after
 * any sequence of calls, -1 if the context has no guard words (the variable was not set at create, or no call has
 * touched the GPU yet).  Errors: E_INVALID (null), E_HIP. */
int adore_check_guards(adore_ctx *ctx, int32_t *damaged);

int adore_abi_version(void);

#ifdef __cplusplus
}
#endif
#endif /* ADORE_H */
