// Host side of the C ABI declared in include/adore.h: argument checks, the
// per-step state machine, the workspace layout and the launch order.
//
// Nothing here waits for the GPU inside a step.  The numbers of occupied slots
// (o), released slots (x) and rebuilt tokens (r) of a step depend only on
// (n, S, K, R), so the host knows every launch shape without reading results
// back:  o = occupied_before + 1,  x = max(0, o - m),  r = min(R, n + 1 - min(o, m)).
//
// Streams.  Attention and the rebuild GEMM run on the caller's stream.  The two selections run on a side stream
// owned by the context, and the controller on a second one: they depend on neither the attention output nor the cache contents.  The
// selections of step n rank the tokens before n, so they wait for the controller of step n-1 (ev_ctrl), not
// for their own step's; the chain of step n+1 runs under the GEMM of step n (and the attention of step n+1).
// The GEMM waits for its own step's selections (ev_join, one event per step: a true dependency).  In the other
// direction there is only a hazard: the selections must not overwrite lists that an attention still reads.
// slot_pos / insert_slot / free_list / rebuilt_pos are therefore rings of kRing copies: the selections of step n
// write copy (n + 1) % kRing, whose last reader was the attention of step n - kRing + 1, and their stream waits
// for the caller's stream only once in kSyncEvery steps: at a step n that is a multiple of kSyncEvery it waits
// for the attention of step n - 2, which covers the steps n .. n + kSyncEvery - 1 as long as
// n + kSyncEvery - 1 - (kRing - 1) <= n - 2.  (Every cross-stream event costs several microseconds on
// the GPU and on the host; with one wait per step in each direction they added up to 9 us per step.)
// Inputs.  The side kernels read what the caller passes to a step (x_n, score_override).  By default
// (adore_set_input_order(ctx, 1)) the side stream therefore starts a step's work behind an event recorded
// on the caller's stream at the top of the call, like any work on the caller's stream itself; the side
// stream then never runs ahead and the periodic wait above is not needed.  A caller whose inputs are
// complete in memory when the call is made switches this off and saves that event.
// ADORE_NO_OVERLAP=1 puts everything on the caller's stream.
#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <new>

#include "adore_internal.h"

using namespace adore;

namespace adore {

ScopedTimer::ScopedTimer(adore_ctx *ctx, int kernel, hipStream_t) : on_(false) {
  ev_[0] = ev_[1] = nullptr;
  if (!ctx->timing) return;
  for (int i = 0; i < 2; ++i) {
    if (!ctx->event_pool.empty()) {
      ev_[i] = ctx->event_pool.back();
      ctx->event_pool.pop_back();
    } else if (hipEventCreate(&ev_[i]) != hipSuccess) {
      return;   // falls back to an untimed launch
    }
  }
  on_ = true;
  ctx->timed.push_back(TimedLaunch{kernel, ev_[0], ev_[1]});
}

}  // namespace adore

namespace {

size_t align_up(size_t v, size_t a = 256) { return (v + a - 1) / a * a; }

struct Layout {
  size_t cache_k, cache_v, slot_pos, score, z, insert_slot, free_list, released_pos, rebuilt_pos, init_res,
      att_part, att_logit, att_ml, gi, zseq, cvec, avec, fwd_q, fwd_o, fwd_x, rope, total;
  std::vector<size_t> guards;   // offsets of the guard words (debug layout), one run behind every region
};

// Debug layout (ADORE_GUARD_WORDS=1 in the environment of the process): every region of the workspace is followed
// by kGuardBytes of a fixed pattern that no kernel ever has a reason to touch; adore_check_guards counts the words
// that changed.  adore_workspace_bytes and adore_create read the variable alike.
constexpr size_t kGuardBytes = 256;
constexpr uint32_t kGuardWord = 0xA5A5A5A5u;
bool guard_words_on() {
  const char *e = getenv("ADORE_GUARD_WORDS");
  return e && atoi(e) != 0;
}

// Upper limits that keep every row, slot and token count of a configuration (and their products, which kernels and
// launch shapes hold in 32-bit integers) far inside the range of int; byte counts are 64-bit throughout.
constexpr int kMaxLayers = 4096, kMaxRows = 1 << 20 /* batch x heads */, kMaxWidth = 1 << 20 /* hidden, H x d */,
              kMaxAnySlots = 1 << 20;

bool config_ok(const adore_config *c) {
  if (!c) return false;
  if (c->layers > kMaxLayers || c->batch > kMaxRows || c->heads > kMaxRows || c->head_dim > kMaxWidth ||
      c->hidden > kMaxWidth || c->cache_slots > kMaxAnySlots || c->max_positions > (1 << 24) || c->ctrl_hidden > kMaxWidth)
    return false;
  if (c->batch > 0 && c->heads > 0 && c->head_dim > 0 &&
      ((long long)c->batch * c->heads > kMaxRows || (long long)c->heads * c->head_dim > kMaxWidth))
    return false;
  return c->layers > 0 && c->batch > 0 && c->heads > 0 && c->head_dim > 0 && c->hidden > 0 &&
         c->cache_slots >= 2 && c->rebuild_budget >= 0 && c->rebuild_budget <= c->cache_slots - 2 &&
         c->max_positions >= 2 && c->ctrl_hidden > 0 && (c->dtype == ADORE_F32 || c->dtype == ADORE_BF16) &&
         (c->score_mode == ADORE_SCORE_STATIC || c->score_mode == ADORE_SCORE_RESCORE ||
          c->score_mode == ADORE_SCORE_H2O) &&
         std::isfinite(c->pos_scale) && std::isfinite(c->rope_base) && c->rope_base >= 0.f;
}

bool config_supported(const adore_config *c) {
  // the selecting release kernel keeps a row's keys in the registers of one wave; a cache that never has to
  // release (K - R - 1 >= N_max: full attention) may have any number of slots
  const bool never_releases = c->cache_slots - c->rebuild_budget - 1 >= c->max_positions;
  if (c->score_mode == ADORE_SCORE_H2O) {
    // scores belong to a layer; the per-sequence choice counts in 8 bits how many heads hold a token and keeps the
    // ranking keys of a sequence in LDS
    if (c->layers != 1 || c->heads > 255 || c->rope_base > 0.f || c->cache_slots > kMaxSlots ||
        h2o_choice_lds_bytes(*c, c->max_positions - 1) > 64 * 1024)
      return false;
  }
  return (c->head_dim == 64 || c->head_dim == 128) && (c->cache_slots <= kMaxSlots || never_releases) &&
         c->hidden % 8 == 0 && c->max_positions <= kMaxPositions && c->ctrl_hidden <= 1024 &&
         (c->score_mode != ADORE_SCORE_RESCORE || c->ctrl_hidden % 4 == 0);
}

Layout make_layout(const adore_config &c) {
  const size_t es = elem_size(c);
  const size_t BH = size_t(c.batch) * c.heads;
  const size_t R1 = size_t(c.rebuild_budget) + 1;
  Layout l;
  size_t off = 0;
  const bool guarded = guard_words_on();
  auto take = [&](size_t bytes) {
    const size_t at = off;
    off = align_up(off + bytes);
    if (guarded) {
      l.guards.push_back(off);
      off += kGuardBytes;
    }
    return at;
  };
  l.cache_k = take(size_t(c.layers) * BH * c.cache_slots * c.head_dim * es);
  l.cache_v = take(size_t(c.layers) * BH * c.cache_slots * c.head_dim * es);
  l.slot_pos = take(kRing * BH * c.cache_slots * 4);
  const bool h2o = c.score_mode == ADORE_SCORE_H2O;
  l.score = take(size_t(c.batch) * (h2o ? c.heads : 1) * c.max_positions * 4);   // H2O: per head
  l.z = take(size_t(c.batch) * c.ctrl_hidden * 4);
  l.insert_slot = take(kRing * align_up(BH * 4));
  l.free_list = take(kRing * align_up(BH * R1 * 4));
  l.released_pos = take(BH * R1 * 4);
  l.rebuilt_pos = take(kRing * align_up(size_t(c.batch) * (c.rebuild_budget > 0 ? c.rebuild_budget : 1) * 4));
  l.init_res = take(size_t(c.batch) * (h2o ? c.heads : 1) * c.cache_slots * 4);
  l.att_part = take(BH * kMaxSplits * (size_t(c.head_dim) + 2) * 4);
  l.att_logit = take(h2o ? BH * c.cache_slots * 4 : 0);
  l.att_ml = take(h2o ? BH * 2 * 4 : 0);
  size_t gi_rows = size_t(c.batch) * kPromptChunk;
  if (gi_rows < size_t(kMaxCtrlSplit) * kCtrlSplitTokens) gi_rows = size_t(kMaxCtrlSplit) * kCtrlSplitTokens;
  l.gi = take(gi_rows * 3 * c.ctrl_hidden * 4);
  l.zseq = take(size_t(c.batch) * kPromptChunk * c.ctrl_hidden * 4);
  const bool rescore = c.score_mode == ADORE_SCORE_RESCORE;
  l.cvec = take(rescore ? size_t(c.batch) * c.max_positions * c.ctrl_hidden * 4 : 0);
  l.avec = take(rescore ? size_t(c.ctrl_hidden) * 4 : 0);
  const size_t fwd_rows = size_t(c.batch) * R1;
  l.fwd_q = take(fwd_rows * c.heads * c.head_dim * es);
  l.fwd_o = take(fwd_rows * c.heads * c.head_dim * es);
  l.fwd_x = take(fwd_rows * c.hidden * es);
  l.rope = take(c.rope_base > 0.f ? size_t(c.max_positions) * (c.head_dim / 2) * 24 : 0);   // fp64 table, fp32 copy
  l.total = off;
  return l;
}

// Launch shape of the attention kernel.  As few splits per (b,h) row as still give every
// compute unit a workgroup (each split costs a partial and, above one, the merge kernel);
// then as many waves per workgroup as leave each wave at least 32 slots.
// ADORE_ATTEND_SPLIT / ADORE_ATTEND_WAVES override the choice (for tuning runs).
void choose_split(adore_ctx *ctx) {
  const adore_config &c = ctx->cfg;
  const int rows = c.batch * c.heads;
  int nsplit = 1;
  while (nsplit < kMaxSplits && rows * nsplit < 256 && c.cache_slots / (nsplit * 2) >= 64) nsplit *= 2;
  if (const char *e = getenv("ADORE_ATTEND_SPLIT")) {
    const int v = atoi(e);
    if (v >= 1 && v <= kMaxSplits) nsplit = v;
  }
  ctx->nsplit = nsplit;
  ctx->chunk = (c.cache_slots + nsplit - 1) / nsplit;
  // measured at B*H = 512 rows: 4 waves 23.8 us, 8 waves 24.8 us at 512 slots per row (16 waves lose to both);
  // 8 waves 105 us, 4 waves 109 us at 4096 rows of 256 slots
  ctx->attend_waves = ctx->chunk >= 512 ? 4 : ctx->chunk >= 256 ? 8 : 4;
  if (const char *e = getenv("ADORE_ATTEND_WAVES")) {
    const int v = atoi(e);
    if (v == 4 || v == 8 || v == 16) ctx->attend_waves = v;
  }
}

#define ADORE_TRY(expr)              \
  do {                               \
    const hipError_t e_ = (expr);    \
    if (e_ != hipSuccess) return ADORE_E_HIP; \
  } while (0)

// The side stream and its events are made on the first call that touches the GPU, so that a
// context can be created (and its host-side checks exercised) on a machine without one.
// The context's events only order its streams against each other on one device: no timing, and no system-scope
// fence (cache write-back and invalidation for the host's and other devices' sake) when they complete.
constexpr unsigned kSyncEventFlags = hipEventDisableTiming | hipEventDisableSystemFence;

// The guard words get their pattern on the first call that touches the GPU (a context can be created without one).
int ensure_guards(adore_ctx *ctx) {
  if (ctx->guards_ready) return ADORE_OK;
  for (size_t off : ctx->guard_off)
    if (hipMemsetAsync(ctx->ws_base + off, int(kGuardWord & 0xff), kGuardBytes, ctx->stream) != hipSuccess) return ADORE_E_HIP;
  ctx->guards_ready = true;
  return ADORE_OK;
}

int ensure_side_stream(adore_ctx *ctx) {
  if (ensure_guards(ctx) != ADORE_OK) return ADORE_E_HIP;
  if (!ctx->overlap || ctx->side_ready) return ADORE_OK;
  bool ok = hipStreamCreateWithFlags(&ctx->side, hipStreamNonBlocking) == hipSuccess;
  ok = ok && hipStreamCreateWithFlags(&ctx->side2, hipStreamNonBlocking) == hipSuccess;
  ok = ok && hipEventCreateWithFlags(&ctx->ev_ctrl, kSyncEventFlags) == hipSuccess;
  ok = ok && hipEventCreateWithFlags(&ctx->ev_att, kSyncEventFlags) == hipSuccess;
  ok = ok && hipEventCreateWithFlags(&ctx->ev_join, kSyncEventFlags) == hipSuccess;
  ok = ok && hipEventCreateWithFlags(&ctx->ev_in, kSyncEventFlags) == hipSuccess;
  if (!ok) {   // leave the context as it was: whatever was made so far goes again
    if (ctx->side != ctx->stream && ctx->side) (void)hipStreamDestroy(ctx->side);
    if (ctx->side2 != ctx->stream && ctx->side2) (void)hipStreamDestroy(ctx->side2);
    for (hipEvent_t *e : {&ctx->ev_ctrl, &ctx->ev_att, &ctx->ev_join, &ctx->ev_in}) {
      if (*e) (void)hipEventDestroy(*e);
      *e = nullptr;
    }
    ctx->side = ctx->side2 = ctx->stream;
    return ADORE_E_HIP;
  }
  ctx->side_ready = true;
  return ADORE_OK;
}

// Ordered inputs: the side stream starts a step's work behind everything the caller's stream holds now.
// selections: the step has work on the selections' stream as well (not when they ride in the attention launch).
hipError_t order_side_after_caller(adore_ctx *ctx, bool selections = true) {
  if (!ctx->overlap || !ctx->ordered) return hipSuccess;
  hipError_t e = hipEventRecord(ctx->ev_in, ctx->stream);
  if (e == hipSuccess && selections) e = hipStreamWaitEvent(ctx->side, ctx->ev_in, 0);
  if (e == hipSuccess && ctx->side2 != ctx->side) e = hipStreamWaitEvent(ctx->side2, ctx->ev_in, 0);
  return e;
}

// Whether the side stream may run ahead of the caller's stream (and so needs the periodic wait of the ring).
bool runs_ahead(const adore_ctx *ctx) { return ctx->overlap && !ctx->ordered; }

// The controller of the current step, on a stream of its own: the selections of the next step wait for it
// (ev_ctrl), those of this step do not queue behind it.  They do not need its score: the current token is exempt
// from release and holds a row.  (In RESCORE mode it also writes the current token's score at distance 0 and the
// vector the later rescorings start from; the tokens before it are rescored on the selections' stream.)
hipError_t launch_controller(adore_ctx *ctx, const void *x_n, int seq_rows, const float *score_override) {
  const adore_config &c = ctx->cfg;
  hipStream_t st = ctx->side2;
  int ksplit = 1;
  hipError_t e = launch_ctrl_input(ctx, st, x_n, c.batch, 1, seq_rows, &ksplit);
  if (e == hipSuccess) e = launch_ctrl_cell(ctx, st, 1, ctx->n, score_override, 1, ksplit);
  if (e == hipSuccess && ctx->overlap) e = hipEventRecord(ctx->ev_ctrl, st);
  return e;
}

void reset_step(adore_ctx *ctx) {
  std::fill(ctx->attended.begin(), ctx->attended.end(), 0);
  std::fill(ctx->rebuilt.begin(), ctx->rebuilt.end(), 0);
  ctx->n_attended = ctx->n_rebuilt = 0;
  ctx->scheduled = false;
  ctx->r_step = 0;
}

}  // namespace

extern "C" {

size_t adore_workspace_bytes(const adore_config *cfg) {
  if (!config_ok(cfg)) return 0;
  return make_layout(*cfg).total;
}

int adore_create(const adore_config *cfg, const adore_weights *weights, void *workspace,
                 size_t workspace_bytes, void *hip_stream, adore_ctx **out) {
  if (!cfg || !weights || !workspace || !out) return ADORE_E_INVALID;
  if (!config_ok(cfg)) return ADORE_E_INVALID;
  if (!weights->w_kv || !weights->gru_w_ih || !weights->gru_w_hh || !weights->gru_b_ih || !weights->gru_b_hh ||
      !weights->pos_w || !weights->pos_b || !weights->mlp_w1 || !weights->mlp_b1 || !weights->out_w ||
      !weights->out_b)
    return ADORE_E_INVALID;
  if (!config_supported(cfg)) return ADORE_E_UNSUPPORTED;
  const Layout l = make_layout(*cfg);
  if (workspace_bytes < l.total || (reinterpret_cast<uintptr_t>(workspace) & 255) != 0) return ADORE_E_WORKSPACE;
  adore_ctx *ctx = new (std::nothrow) adore_ctx();
  if (!ctx) return ADORE_E_INVALID;
  ctx->cfg = *cfg;
  ctx->w = *weights;
  ctx->stream = static_cast<hipStream_t>(hip_stream);
  char *base = static_cast<char *>(workspace);
  ctx->cache_k = base + l.cache_k;
  ctx->cache_v = base + l.cache_v;
  const size_t BH = size_t(cfg->batch) * cfg->heads;
  const size_t R1 = size_t(cfg->rebuild_budget) + 1;
  const size_t Rdim = cfg->rebuild_budget > 0 ? cfg->rebuild_budget : 1;
  for (int i = 0; i < kRing; ++i) {
    ctx->slot_pos[i] = reinterpret_cast<int32_t *>(base + l.slot_pos + i * BH * cfg->cache_slots * 4);
    ctx->insert_slot[i] = reinterpret_cast<int32_t *>(base + l.insert_slot + i * align_up(BH * 4));
    ctx->free_list[i] = reinterpret_cast<int32_t *>(base + l.free_list + i * align_up(BH * R1 * 4));
    ctx->rebuilt_pos[i] = reinterpret_cast<int32_t *>(base + l.rebuilt_pos + i * align_up(size_t(cfg->batch) * Rdim * 4));
  }
  ctx->score = reinterpret_cast<float *>(base + l.score);
  ctx->z = reinterpret_cast<float *>(base + l.z);
  ctx->released_pos = reinterpret_cast<int32_t *>(base + l.released_pos);
  ctx->init_res = reinterpret_cast<int32_t *>(base + l.init_res);
  ctx->att_part = reinterpret_cast<float *>(base + l.att_part);
  ctx->att_logit = reinterpret_cast<float *>(base + l.att_logit);
  ctx->att_ml = reinterpret_cast<float *>(base + l.att_ml);
  ctx->gi = reinterpret_cast<float *>(base + l.gi);
  ctx->zseq = reinterpret_cast<float *>(base + l.zseq);
  ctx->cvec = reinterpret_cast<float *>(base + l.cvec);
  ctx->avec = reinterpret_cast<float *>(base + l.avec);
  ctx->fwd_q = base + l.fwd_q;
  ctx->fwd_o = base + l.fwd_o;
  ctx->fwd_x = base + l.fwd_x;
  ctx->rope = base + l.rope;
  ctx->rope_f = reinterpret_cast<float2 *>(base + l.rope + size_t(cfg->max_positions) * (cfg->head_dim / 2) * 16);
  ctx->ws_base = base;
  ctx->guard_off = l.guards;
  ctx->guards_ready = false;
  ctx->forward = false;
  ctx->r_pending = 0;
  ctx->ins_stride = 1;
  ctx->ins_off = 0;
  ctx->ins_from_list = false;
  ctx->rode = false;
  ctx->inited = false;
  ctx->n = 0;
  ctx->occ = 0;
  ctx->cur = 0;
  const char *no = getenv("ADORE_NO_OVERLAP");
  // H2O scores come out of the step's own attention: its selections follow it on the caller's stream, and there
  // is no controller to run beside them
  ctx->overlap = !(no && atoi(no) != 0) && cfg->score_mode != ADORE_SCORE_H2O;
  const char *nr = getenv("ADORE_NO_RIDE");
  ctx->ride = ctx->overlap && !(nr && atoi(nr) != 0);
  // Whether the selections may ride in the attention launch: static scores, a cache that releases, and the role's
  // LDS at the last step of the longest sequence (its need grows with n) within what a workgroup gets without
  // asking for more, 64 KB, next to the attention kernel's own static LDS.  Decided once, here, so that no step
  // in the middle of a sequence finds its launch refused.
  ctx->ride_fits = cfg->score_mode == ADORE_SCORE_STATIC && cfg->cache_slots <= kMaxSlots &&
                   riding_lds_bytes(cfg->max_positions - 1, cfg->cache_slots, cfg->rebuild_budget) + kAttendStaticLds <=
                       64 * 1024;
  ctx->side = ctx->side2 = ctx->stream;
  ctx->ev_ctrl = nullptr;
  ctx->ev_att = ctx->ev_join = ctx->ev_in = nullptr;
  ctx->ordered = true;
  ctx->steps_done = 0;
  ctx->side_ready = false;
  ctx->attended.assign(cfg->layers, 0);
  ctx->rebuilt.assign(cfg->layers, 0);
  ctx->timing = false;
  reset_step(ctx);
  choose_split(ctx);
  *out = ctx;
  return ADORE_OK;
}

int adore_destroy(adore_ctx *ctx) {
  if (!ctx) return ADORE_E_INVALID;
  for (auto &t : ctx->timed) {
    (void)hipEventDestroy(t.start);
    (void)hipEventDestroy(t.stop);
  }
  for (auto &e : ctx->event_pool) (void)hipEventDestroy(e);
  if (ctx->overlap && ctx->side_ready) {
    (void)hipStreamSynchronize(ctx->side);
    (void)hipStreamSynchronize(ctx->side2);
    (void)hipStreamDestroy(ctx->side);
    (void)hipStreamDestroy(ctx->side2);
    for (hipEvent_t e : {ctx->ev_att, ctx->ev_join, ctx->ev_in, ctx->ev_ctrl})
      if (e) (void)hipEventDestroy(e);
  }
  delete ctx;
  return ADORE_OK;
}

int adore_init_cache(adore_ctx *ctx, const void *prompt_k, const void *prompt_v, const void *hidden_store,
                     const void *ctrl_input, const float *score_override, int32_t S) {
  if (!ctx || !prompt_k || !prompt_v || !ctrl_input) return ADORE_E_INVALID;
  const adore_config &c = ctx->cfg;
  if (S < 1 || S >= c.max_positions) return ADORE_E_INVALID;
  const bool forward = hidden_store == nullptr;
  if (forward && c.cache_slots > fwd_attend_max_slots()) return ADORE_E_UNSUPPORTED;
  const bool rescore = c.score_mode == ADORE_SCORE_RESCORE;
  if (rescore && score_override) return ADORE_E_INVALID;   // scores are recomputed at every step
  if (h2o_mode(ctx) && forward) return ADORE_E_UNSUPPORTED;
  const size_t es = elem_size(c);
  const int m = c.cache_slots - c.rebuild_budget - 1;
  const int keep = S < m ? S : m;
  const int pool = S - keep;
  const int r0 = pool < c.rebuild_budget ? pool : c.rebuild_budget;

  // init runs on the caller's stream only; anything a previous job left on the side stream ends first
  if (ensure_side_stream(ctx) != ADORE_OK) return ADORE_E_HIP;
  if (ctx->overlap) {
    ADORE_TRY(hipStreamSynchronize(ctx->side));
    ADORE_TRY(hipStreamSynchronize(ctx->side2));
  }
  hipStream_t st = ctx->stream;
  ctx->cur = 0;
  if (h2o_mode(ctx)) {
    // the prompt's scores are given (or zero); every head picks its own residents, then the per-sequence choice
    ADORE_TRY(launch_h2o_init_scores(ctx, score_override, S));
    ADORE_TRY(launch_h2o_init_select(ctx, ctx->cur, ctx->cur + 1, S, keep));
    ADORE_TRY(launch_h2o_choice(ctx, ctx->cur, ctx->cur + 1, S - 1, nullptr, nullptr));
    ADORE_TRY(launch_init_copy(ctx, prompt_k, prompt_v, S, keep));
    if (pool > 0) ADORE_TRY(launch_rebuild_gemm(ctx, 0, hidden_store, ctx->cur + 1, c.rebuild_budget));
    ctx->steps_done = 0;
    ctx->n = S;
    ctx->occ = 0;
    ctx->inited = true;
    ctx->forward = false;
    ctx->r_pending = 0;
    ctx->ins_stride = 1;
    ctx->ins_off = 0;
    ctx->ins_from_list = false;
    ctx->rode = false;
    reset_step(ctx);
    return ADORE_OK;
  }
  ADORE_TRY(launch_rope_table(ctx));
  // controller over the prompt: z_{-1} = 0, tokens in order, in chunks
  ADORE_TRY(launch_fill_i32(ctx, reinterpret_cast<int32_t *>(ctx->z), 0, size_t(c.batch) * c.ctrl_hidden));
  for (int i0 = 0; i0 < S; i0 += kPromptChunk) {
    const int len = (S - i0 < kPromptChunk) ? S - i0 : kPromptChunk;
    const char *x = static_cast<const char *>(ctrl_input) + size_t(i0) * c.hidden * es;
    int ksplit = 1;
    ADORE_TRY(launch_ctrl_input(ctx, st, x, c.batch * len, len, S, &ksplit));
    ADORE_TRY(launch_ctrl_cell(ctx, st, len, i0, score_override ? score_override + i0 : nullptr, S, ksplit));
  }
  if (rescore) {   // every prompt token as seen from the last one
    ADORE_TRY(launch_ctrl_avec(ctx, st));
    ADORE_TRY(launch_rescore(ctx, st, S - 1, S - 1));
  }
  // slot map and reserved slot go to copy `cur`, the rebuild lists to `cur + 1` (where a step's GEMM reads
  // them); for the forward, whose first step rebuilds these tokens itself, the lists go to `cur` as well
  ADORE_TRY(launch_init_select(ctx, ctx->cur, forward ? ctx->cur : ctx->cur + 1, S, keep, r0));
  ADORE_TRY(launch_init_copy(ctx, prompt_k, prompt_v, S, keep));
  const size_t hs_layer = size_t(c.batch) * c.max_positions * c.hidden * es;
  for (int l = 0; l < c.layers && !forward; ++l) {
    ADORE_TRY(launch_rebuild_gemm(ctx, l, static_cast<const char *>(hidden_store) + l * hs_layer, ctx->cur + 1, r0));
  }
  if (ctx->overlap) ADORE_TRY(hipEventRecord(ctx->ev_att, st));   // the first selections wait for everything above
  ctx->steps_done = 0;
  if (ctx->overlap) {   // what the first step waits for is all above
    ADORE_TRY(hipEventRecord(ctx->ev_join, st));
    ADORE_TRY(hipEventRecord(ctx->ev_ctrl, st));
    // The side streams start behind the init whatever the input order: the first step's controller reads the GRU
    // state the prompt scan leaves and reuses its scratch, the first selections read the slot map.  (With ordered
    // inputs every step waits for the caller's stream anyway; without, nothing else would hold them back.)
    ADORE_TRY(hipStreamWaitEvent(ctx->side2, ctx->ev_ctrl, 0));
    ADORE_TRY(hipStreamWaitEvent(ctx->side, ctx->ev_ctrl, 0));
  }
  ctx->n = S;
  ctx->occ = keep + r0;
  ctx->inited = true;
  ctx->forward = forward;
  ctx->r_pending = r0;
  ctx->ins_stride = 1;
  ctx->ins_off = 0;
  ctx->ins_from_list = false;
  ctx->rode = false;
  reset_step(ctx);
  return ADORE_OK;
}

namespace {

// The three stages without the order checks (the public calls do those).

int do_attend(adore_ctx *ctx, int32_t layer, const void *q, const void *k_new, const void *v_new, float *out) {
  ADORE_TRY(launch_attend(ctx, layer, q, k_new, v_new, out));
  ctx->attended[layer] = 1;
  if (++ctx->n_attended == ctx->cfg.layers && runs_ahead(ctx) && (ctx->steps_done + 2) % kSyncEvery == 0) {
    ADORE_TRY(hipEventRecord(ctx->ev_att, ctx->stream));   // what the side stream waits for two steps from now
  }
  return ADORE_OK;
}

int do_schedule(adore_ctx *ctx, const void *x_n, const float *score_override, int32_t *slot_map,
                int32_t *released_pos, int32_t *rebuilt_pos) {
  const adore_config &c = ctx->cfg;
  if (h2o_mode(ctx)) {
    // The step's attention is added to the scores, every head releases on its own (how many rows, it counts
    // itself), then the per-sequence choice.  Tokens exist to be rebuilt once some head has had to give one up,
    // which cannot happen before there are more tokens than persistent rows; how many are chosen is decided on
    // the device, and the GEMM skips the ranks that stay empty.
    const int dst = (ctx->cur + 1) % kRing;
    ADORE_TRY(launch_h2o_release(ctx, ctx->cur, dst, slot_map, released_pos));
    ADORE_TRY(launch_h2o_choice(ctx, dst, dst, ctx->n, slot_map, rebuilt_pos));
    ctx->scheduled = true;
    ctx->r_step = ctx->n + 1 > c.cache_slots - c.rebuild_budget - 1 ? c.rebuild_budget : 0;
    return ADORE_OK;
  }
  const int m = c.cache_slots - c.rebuild_budget - 1;
  const int o = ctx->occ + 1;
  const int x = o > m ? o - m : 0;
  const int kept = o - x;
  const int pool = ctx->n + 1 - kept;
  const int r = pool < c.rebuild_budget ? pool : c.rebuild_budget;
  const int src = ctx->cur, dst = (ctx->cur + 1) % kRing;
  hipStream_t st = ctx->side;
  ADORE_TRY(order_side_after_caller(ctx));
  if (ctx->rode && runs_ahead(ctx)) {
    // the steps before this one ran their selections on the caller's stream: the side stream catches up once
    ADORE_TRY(hipEventRecord(ctx->ev_att, ctx->stream));
    ADORE_TRY(hipStreamWaitEvent(st, ctx->ev_att, 0));
    ctx->steps_done = 1;   // the next regular wait is due at a multiple of kSyncEvery, covered by this one until then
  }
  ctx->rode = false;

  // the selections rank the tokens before the current one: they wait for the previous step's controller, not for
  // this step's (which touches only its own state and the score array and may run as early as its inputs allow)
  if (ctx->overlap) ADORE_TRY(hipStreamWaitEvent(st, ctx->ev_ctrl, 0));
  ADORE_TRY(launch_controller(ctx, x_n, 1, score_override));
  if (c.score_mode == ADORE_SCORE_RESCORE) ADORE_TRY(launch_rescore(ctx, st, ctx->n, ctx->n - 1));
  // copy `dst` was `cur` kRing - 1 steps ago: see the note on the ring at the top of this file
  if (runs_ahead(ctx) && ctx->steps_done % kSyncEvery == 0) ADORE_TRY(hipStreamWaitEvent(st, ctx->ev_att, 0));
  ADORE_TRY(launch_release(ctx, st, src, dst, x, slot_map, released_pos));
  ADORE_TRY(launch_rebuild_select(ctx, st, dst, r, slot_map, rebuilt_pos));
  if (ctx->overlap) ADORE_TRY(hipEventRecord(ctx->ev_join, st));
  ctx->scheduled = true;
  ctx->r_step = r;
  ctx->occ = kept + r;
  return ADORE_OK;
}

int do_rebuild(adore_ctx *ctx, int32_t layer, const void *hidden_store_layer) {
  if (ctx->n_rebuilt == 0 && ctx->overlap) {
    // from here on the caller's stream sees everything the selections wrote, outputs included
    ADORE_TRY(hipStreamWaitEvent(ctx->stream, ctx->ev_join, 0));
  }
  ADORE_TRY(launch_rebuild_gemm(ctx, layer, hidden_store_layer, (ctx->cur + 1) % kRing, ctx->r_step));
  ctx->rebuilt[layer] = 1;
  if (++ctx->n_rebuilt == ctx->cfg.layers) {
    ctx->n++;
    ctx->steps_done++;
    ctx->cur = (ctx->cur + 1) % kRing;
    ctx->ins_stride = 1;       // this step's per-sequence choice wrote insert_slot
    ctx->ins_off = 0;
    ctx->ins_from_list = false;
    reset_step(ctx);
  }
  return ADORE_OK;
}

// The whole step of one layer with the two selections riding in the attention launch (static score mode).
// Neither selection of step n looks at the current token's score, so only the controller stays on a side
// stream; what it writes (the score of token n) is first needed by the selections of step n+1, which is
// what the one wait at the top is for.  No other event, and no kernel of the selections runs next to the GEMM.
int do_ridden_step(adore_ctx *ctx, const void *q, const void *k_new, const void *v_new, const void *hidden_store,
                   const void *x_n, const float *score_override, float *out, int32_t *slot_map) {
  const adore_config &c = ctx->cfg;
  const int m = c.cache_slots - c.rebuild_budget - 1;
  const int o = ctx->occ + 1;
  const int x = o > m ? o - m : 0;
  const int kept = o - x;
  const int pool = ctx->n + 1 - kept;
  const int r = pool < c.rebuild_budget ? pool : c.rebuild_budget;
  const int dst = (ctx->cur + 1) % kRing;
  ADORE_TRY(order_side_after_caller(ctx, false));
  ADORE_TRY(hipStreamWaitEvent(ctx->stream, ctx->ev_ctrl, 0));   // the controller of the step before
  ADORE_TRY(launch_controller(ctx, x_n, 1, score_override));
  RidingSelections sel;
  sel.dst = dst; sel.x = x; sel.r = r;
  sel.map_out = slot_map; sel.rel_out = nullptr; sel.rb_out = nullptr;
  ADORE_TRY(launch_attend(ctx, 0, q, k_new, v_new, out, &sel));
  ADORE_TRY(launch_rebuild_gemm(ctx, 0, hidden_store, dst, r, ctx->slot_pos[dst], slot_map));
  ctx->occ = kept + r;
  ctx->n++;
  ctx->steps_done++;
  ctx->cur = dst;
  ctx->ins_stride = c.rebuild_budget + 1;   // the slot behind the rebuilt tokens' slots in the free list
  ctx->ins_off = r;
  ctx->ins_from_list = true;
  ctx->rode = true;
  reset_step(ctx);
  return ADORE_OK;
}

}  // namespace

int adore_attend(adore_ctx *ctx, int32_t layer, const void *q, const void *k_new, const void *v_new,
                 float *out) {
  if (!ctx || !q || !k_new || !v_new || !out) return ADORE_E_INVALID;
  if (layer < 0 || layer >= ctx->cfg.layers) return ADORE_E_INVALID;
  if (!ctx->inited || ctx->forward || ctx->scheduled || ctx->attended[layer] || ctx->n >= ctx->cfg.max_positions)
    return ADORE_E_STATE;
  return do_attend(ctx, layer, q, k_new, v_new, out);
}

int adore_schedule(adore_ctx *ctx, const void *x_n, const float *score_override, int32_t *slot_map,
                   int32_t *released_pos, int32_t *rebuilt_pos) {
  if (!ctx || (!x_n && !h2o_mode(ctx))) return ADORE_E_INVALID;
  if (score_override && ctx->cfg.score_mode != ADORE_SCORE_STATIC) return ADORE_E_INVALID;
  if (!ctx->inited || ctx->forward || ctx->scheduled || ctx->n_attended != ctx->cfg.layers) return ADORE_E_STATE;
  return do_schedule(ctx, x_n, score_override, slot_map, released_pos, rebuilt_pos);
}

int adore_rebuild(adore_ctx *ctx, int32_t layer, const void *hidden_store_layer) {
  if (!ctx || !hidden_store_layer) return ADORE_E_INVALID;
  if (layer < 0 || layer >= ctx->cfg.layers) return ADORE_E_INVALID;
  if (!ctx->inited || ctx->forward || !ctx->scheduled || ctx->rebuilt[layer]) return ADORE_E_STATE;
  return do_rebuild(ctx, layer, hidden_store_layer);
}

int adore_decode_step(adore_ctx *ctx, const void *q, const void *k_new, const void *v_new,
                      const void *hidden_store, const void *x_n, const float *score_override, float *out,
                      int32_t *slot_map) {
  if (!ctx || !q || !k_new || !v_new || !hidden_store || (!x_n && !h2o_mode(ctx)) || !out) return ADORE_E_INVALID;
  if (ctx->cfg.layers != 1) return ADORE_E_INVALID;
  if (score_override && ctx->cfg.score_mode != ADORE_SCORE_STATIC) return ADORE_E_INVALID;
  if (!ctx->inited || ctx->forward || ctx->scheduled || ctx->n_attended != 0 || ctx->n >= ctx->cfg.max_positions)
    return ADORE_E_STATE;
  if (ctx->ride && ctx->ride_fits) {
    if (ensure_side_stream(ctx) != ADORE_OK) return ADORE_E_HIP;
    return do_ridden_step(ctx, q, k_new, v_new, hidden_store, x_n, score_override, out, slot_map);
  }
  if (h2o_mode(ctx)) {   // the selections need this step's attention
    int rc = do_attend(ctx, 0, q, k_new, v_new, out);
    if (rc != ADORE_OK) return rc;
    rc = do_schedule(ctx, x_n, score_override, slot_map, nullptr, nullptr);
    if (rc != ADORE_OK) return rc;
    return do_rebuild(ctx, 0, hidden_store);
  }
  // The selections do not depend on this step's attention: enqueue them first so that they start
  // while the previous step's GEMM is still running.
  int rc = do_schedule(ctx, x_n, score_override, slot_map, nullptr, nullptr);
  if (rc != ADORE_OK) return rc;
  rc = do_attend(ctx, 0, q, k_new, v_new, out);
  if (rc != ADORE_OK) return rc;
  return do_rebuild(ctx, 0, hidden_store);
}

int adore_forward_step(adore_ctx *ctx, const adore_forward_weights *fw, const void *embed,
                       const float *score_override, void *rows_out, void *layer_rows, int32_t *slot_map,
                       int32_t *released_pos, int32_t *rebuilt_pos) {
  if (!ctx || !fw || !fw->w_q || !fw->w_o || !embed || !rows_out) return ADORE_E_INVALID;
  if (score_override && ctx->cfg.score_mode == ADORE_SCORE_RESCORE) return ADORE_E_INVALID;
  if (!ctx->inited || !ctx->forward || ctx->n >= ctx->cfg.max_positions) return ADORE_E_STATE;
  const adore_config &c = ctx->cfg;
  const int r = ctx->r_pending;              // rows: r rebuilt tokens + the current one, per sequence
  const int Hd = c.heads * c.head_dim;
  const size_t es = elem_size(c);
  // everything the layers read (slot map, slots of the rebuilt tokens and of the current one) was written
  // by the previous step's selections
  ADORE_TRY(order_side_after_caller(ctx));
  if (ctx->overlap) ADORE_TRY(hipStreamWaitEvent(ctx->stream, ctx->ev_join, 0));
  // this step's controller and selections: they read the same lists and write the other buffer, so they
  // run on the side stream next to the layers
  const char *x_n = static_cast<const char *>(embed) + size_t(ctx->n) * c.hidden * es;
  {
    const int m = c.cache_slots - c.rebuild_budget - 1;
    const int o = ctx->occ + 1;
    const int x = o > m ? o - m : 0;
    const int kept = o - x;
    const int pool = ctx->n + 1 - kept;
    const int r_next = pool < c.rebuild_budget ? pool : c.rebuild_budget;
    const int src = ctx->cur, dst = (ctx->cur + 1) % kRing;
    hipStream_t st = ctx->side;
    if (ctx->overlap) ADORE_TRY(hipStreamWaitEvent(st, ctx->ev_ctrl, 0));   // the previous step's controller
    ADORE_TRY(launch_controller(ctx, x_n, c.max_positions, score_override));
    if (c.score_mode == ADORE_SCORE_RESCORE) ADORE_TRY(launch_rescore(ctx, st, ctx->n, ctx->n - 1));
    if (runs_ahead(ctx) && ctx->steps_done % kSyncEvery == 0) ADORE_TRY(hipStreamWaitEvent(st, ctx->ev_att, 0));   // see the note on the ring
    ADORE_TRY(launch_release(ctx, st, src, dst, x, slot_map, released_pos));
    ADORE_TRY(launch_rebuild_select(ctx, st, dst, r_next, slot_map, rebuilt_pos));
    if (ctx->overlap) ADORE_TRY(hipEventRecord(ctx->ev_join, st));
    ctx->r_step = r_next;
    ctx->occ = kept + r_next;
  }
  const char *wq = static_cast<const char *>(fw->w_q);
  const char *wo = static_cast<const char *>(fw->w_o);
  for (int l = 0; l < c.layers; ++l) {
    const void *x_rows = l == 0 ? embed : ctx->fwd_x;
    const bool by_pos = l == 0;
    const bool last = l == c.layers - 1;
    ADORE_TRY(launch_fwd_qkv(ctx, l, wq + size_t(l) * Hd * c.hidden * es, x_rows, by_pos, r));
    ADORE_TRY(launch_fwd_attend(ctx, l, r));
    if (last && runs_ahead(ctx) && (ctx->steps_done + 2) % kSyncEvery == 0) ADORE_TRY(hipEventRecord(ctx->ev_att, ctx->stream));
    ADORE_TRY(launch_fwd_oproj(ctx, wo + size_t(l) * c.hidden * Hd * es, x_rows, by_pos, last ? rows_out : ctx->fwd_x,
                               last ? c.rebuild_budget + 1 : r + 1, last ? c.rebuild_budget : r, r));
    if (layer_rows) {   // the caller's copy of the rows leaving this layer, in the layout of rows_out
      const size_t row = size_t(c.hidden) * es, seq = row * (c.rebuild_budget + 1);
      char *dst = static_cast<char *>(layer_rows) + size_t(l) * c.batch * seq;
      if (last) {
        ADORE_TRY(hipMemcpyAsync(dst, rows_out, size_t(c.batch) * seq, hipMemcpyDeviceToDevice, ctx->stream));
      } else {
        const char *src = static_cast<const char *>(ctx->fwd_x);
        if (r > 0)
          ADORE_TRY(hipMemcpy2DAsync(dst, seq, src, row * (r + 1), row * r, c.batch, hipMemcpyDeviceToDevice, ctx->stream));
        ADORE_TRY(hipMemcpy2DAsync(dst + row * c.rebuild_budget, seq, src + row * r, row * (r + 1), row, c.batch,
                                   hipMemcpyDeviceToDevice, ctx->stream));
      }
    }
  }
  ctx->r_pending = ctx->r_step;
  ctx->n++;
  ctx->steps_done++;
  ctx->cur = (ctx->cur + 1) % kRing;
  reset_step(ctx);
  return ADORE_OK;
}

int adore_get_state(adore_ctx *ctx, int32_t *slot_pos, float *scores, float *z, void *cache_k, void *cache_v,
                    int32_t *step) {
  if (!ctx) return ADORE_E_INVALID;
  if (!ctx->inited || ctx->scheduled || ctx->n_attended != 0) return ADORE_E_STATE;
  const adore_config &c = ctx->cfg;
  const size_t BH = size_t(c.batch) * c.heads;
  const size_t cache_bytes = size_t(c.layers) * BH * c.cache_slots * c.head_dim * elem_size(c);
  if (step) *step = ctx->n;
  if (ctx->overlap && ctx->side_ready) {   // the last selections and the controller's last score
    ADORE_TRY(hipStreamWaitEvent(ctx->stream, ctx->ev_join, 0));
    ADORE_TRY(hipStreamWaitEvent(ctx->stream, ctx->ev_ctrl, 0));
  }
  if (slot_pos)
    ADORE_TRY(hipMemcpyAsync(slot_pos, ctx->slot_pos[ctx->cur], BH * c.cache_slots * 4, hipMemcpyDeviceToDevice,
                             ctx->stream));
  if (scores)
    ADORE_TRY(hipMemcpyAsync(scores, ctx->score, size_t(c.batch) * (h2o_mode(ctx) ? c.heads : 1) * c.max_positions * 4,
                             hipMemcpyDeviceToDevice, ctx->stream));
  if (z && !h2o_mode(ctx))   // no controller, no GRU state
    ADORE_TRY(hipMemcpyAsync(z, ctx->z, size_t(c.batch) * c.ctrl_hidden * 4, hipMemcpyDeviceToDevice, ctx->stream));
  if (cache_k) ADORE_TRY(hipMemcpyAsync(cache_k, ctx->cache_k, cache_bytes, hipMemcpyDeviceToDevice, ctx->stream));
  if (cache_v) ADORE_TRY(hipMemcpyAsync(cache_v, ctx->cache_v, cache_bytes, hipMemcpyDeviceToDevice, ctx->stream));
  return ADORE_OK;
}

int adore_set_state(adore_ctx *ctx, const int32_t *slot_pos, const float *scores, const float *z,
                    const void *cache_k, const void *cache_v, int32_t step) {
  if (!ctx || !slot_pos) return ADORE_E_INVALID;
  const adore_config &c = ctx->cfg;
  if (c.score_mode != ADORE_SCORE_STATIC) return ADORE_E_UNSUPPORTED;   // rescore: the per-token vectors are not part of a
                                                                         // snapshot; H2O: heads differ in what they hold
  if (step < 1 || step >= c.max_positions) return ADORE_E_INVALID;
  if (ctx->scheduled || ctx->n_attended != 0 || ctx->forward) return ADORE_E_STATE;
  const size_t BH = size_t(c.batch) * c.heads;
  const size_t cache_bytes = size_t(c.layers) * BH * c.cache_slots * c.head_dim * elem_size(c);
  if (ensure_side_stream(ctx) != ADORE_OK) return ADORE_E_HIP;
  if (ctx->overlap) {
    ADORE_TRY(hipStreamSynchronize(ctx->side));
    ADORE_TRY(hipStreamSynchronize(ctx->side2));
  }
  // count the occupied slots and find the reserved slot of every row on the host
  std::vector<int32_t> host(BH * c.cache_slots);
  ADORE_TRY(hipMemcpyAsync(host.data(), slot_pos, host.size() * 4, hipMemcpyDeviceToHost, ctx->stream));
  ADORE_TRY(hipStreamSynchronize(ctx->stream));
  std::vector<int32_t> ins(BH);
  int occ = -1;
  for (size_t row = 0; row < BH; ++row) {
    int cnt = 0, first_free = -1;
    for (int k = 0; k < c.cache_slots; ++k) {
      const int32_t p = host[row * c.cache_slots + k];
      if (p >= step) return ADORE_E_INVALID;
      if (p >= 0) cnt++;
      else if (first_free < 0) first_free = k;
    }
    if (first_free < 0) return ADORE_E_INVALID;
    if (occ < 0) occ = cnt;
    if (cnt != occ) return ADORE_E_INVALID;   // uniform policy: same occupancy everywhere
    ins[row] = first_free;
  }
  // uniform policy: every head of a sequence holds the same positions (the per-sequence choice of the tokens to
  // rebuild reads which ones from head 0 alone), each of them once
  {
    std::vector<int32_t> ref, mine;
    for (int b = 0; b < c.batch; ++b) {
      for (int h = 0; h < c.heads; ++h) {
        const int32_t *rowp = host.data() + (size_t(b) * c.heads + h) * c.cache_slots;
        std::vector<int32_t> &v = h == 0 ? ref : mine;
        v.clear();
        for (int k = 0; k < c.cache_slots; ++k)
          if (rowp[k] >= 0) v.push_back(rowp[k]);
        std::sort(v.begin(), v.end());
        if (std::adjacent_find(v.begin(), v.end()) != v.end()) return ADORE_E_INVALID;
        if (h > 0 && mine != ref) return ADORE_E_INVALID;
      }
    }
  }
  ADORE_TRY(hipMemcpyAsync(ctx->slot_pos[ctx->cur], slot_pos, BH * c.cache_slots * 4, hipMemcpyDeviceToDevice,
                           ctx->stream));
  ADORE_TRY(hipMemcpyAsync(ctx->insert_slot[ctx->cur], ins.data(), BH * 4, hipMemcpyHostToDevice, ctx->stream));
  if (scores)
    ADORE_TRY(hipMemcpyAsync(ctx->score, scores, size_t(c.batch) * c.max_positions * 4, hipMemcpyDeviceToDevice,
                             ctx->stream));
  if (z)
    ADORE_TRY(hipMemcpyAsync(ctx->z, z, size_t(c.batch) * c.ctrl_hidden * 4, hipMemcpyDeviceToDevice, ctx->stream));
  if (cache_k) ADORE_TRY(hipMemcpyAsync(ctx->cache_k, cache_k, cache_bytes, hipMemcpyDeviceToDevice, ctx->stream));
  if (cache_v) ADORE_TRY(hipMemcpyAsync(ctx->cache_v, cache_v, cache_bytes, hipMemcpyDeviceToDevice, ctx->stream));
  ADORE_TRY(launch_rope_table(ctx));              // a context restored without an init has none yet
  ADORE_TRY(hipStreamSynchronize(ctx->stream));   // `ins` lives on this stack frame
  if (ctx->overlap) ADORE_TRY(hipEventRecord(ctx->ev_att, ctx->stream));   // the next selections may start at once
  ctx->steps_done = 0;
  ctx->n = step;
  ctx->occ = occ;
  ctx->inited = true;
  ctx->ins_stride = 1;
  ctx->ins_off = 0;
  ctx->ins_from_list = false;
  ctx->rode = false;
  reset_step(ctx);
  return ADORE_OK;
}

int adore_set_input_order(adore_ctx *ctx, int32_t ordered) {
  if (!ctx) return ADORE_E_INVALID;
  if (ctx->scheduled || ctx->n_attended != 0) return ADORE_E_STATE;
  const bool on = ordered != 0;
  if (on == ctx->ordered) return ADORE_OK;
  if (!on && ctx->overlap && ctx->side_ready) {
    // from here on the side stream runs ahead again: start its periodic wait like after an init
    ADORE_TRY(hipEventRecord(ctx->ev_att, ctx->stream));
    ADORE_TRY(hipStreamWaitEvent(ctx->side, ctx->ev_att, 0));
    ADORE_TRY(hipStreamWaitEvent(ctx->side2, ctx->ev_att, 0));
    ctx->steps_done = 0;
    ctx->rode = false;
  }
  ctx->ordered = on;
  return ADORE_OK;
}

int adore_check_guards(adore_ctx *ctx, int32_t *damaged) {
  if (!ctx || !damaged) return ADORE_E_INVALID;
  if (ctx->guard_off.empty() || !ctx->guards_ready) {
    *damaged = -1;
    return ADORE_OK;
  }
  ADORE_TRY(hipStreamSynchronize(ctx->stream));
  if (ctx->overlap && ctx->side_ready) {
    ADORE_TRY(hipStreamSynchronize(ctx->side));
    ADORE_TRY(hipStreamSynchronize(ctx->side2));
  }
  std::vector<uint32_t> host(kGuardBytes / 4);
  int32_t bad = 0;
  for (size_t off : ctx->guard_off) {
    ADORE_TRY(hipMemcpy(host.data(), ctx->ws_base + off, kGuardBytes, hipMemcpyDeviceToHost));
    for (uint32_t w : host) bad += w != kGuardWord;
  }
  *damaged = bad;
  return ADORE_OK;
}

int adore_set_timing(adore_ctx *ctx, int32_t enable) {
  if (!ctx) return ADORE_E_INVALID;
  ctx->timing = enable != 0;
  return ADORE_OK;
}

int adore_read_timing(adore_ctx *ctx, float *ms, int32_t *launches) {
  if (!ctx || !ms || !launches) return ADORE_E_INVALID;
  ADORE_TRY(hipStreamSynchronize(ctx->stream));
  if (ctx->overlap && ctx->side_ready) {
    ADORE_TRY(hipStreamSynchronize(ctx->side));
    ADORE_TRY(hipStreamSynchronize(ctx->side2));
  }
  for (int i = 0; i < ADORE_N_KERNELS; ++i) {
    ms[i] = 0.f;
    launches[i] = 0;
  }
  for (auto &t : ctx->timed) {
    float e = 0.f;
    if (hipEventElapsedTime(&e, t.start, t.stop) == hipSuccess) {
      ms[t.kernel] += e;
      launches[t.kernel]++;
    }
    ctx->event_pool.push_back(t.start);
    ctx->event_pool.push_back(t.stop);
  }
  ctx->timed.clear();
  return ADORE_OK;
}

const char *adore_kernel_name(int32_t kernel) {
  switch (kernel) {
    case ADORE_KERNEL_ATTEND: return "attend";
    case ADORE_KERNEL_ATTEND_COMBINE: return "attend_combine";
    case ADORE_KERNEL_CTRL_INPUT: return "ctrl_input";
    case ADORE_KERNEL_CTRL_CELL: return "ctrl_cell";
    case ADORE_KERNEL_RELEASE: return "release";
    case ADORE_KERNEL_REBUILD_SELECT: return "rebuild_select";
    case ADORE_KERNEL_REBUILD_GEMM: return "rebuild_gemm";
    case ADORE_KERNEL_RESCORE: return "rescore";
    case ADORE_KERNEL_FWD_QKV: return "fwd_qkv";
    case ADORE_KERNEL_FWD_QKV_CUR: return "fwd_qkv_cur";
    case ADORE_KERNEL_FWD_ATTEND: return "fwd_attend";
    case ADORE_KERNEL_FWD_OPROJ: return "fwd_oproj";
    case ADORE_KERNEL_FWD_OPROJ_CUR: return "fwd_oproj_cur";
    case ADORE_KERNEL_ROPE: return "rope";
    case ADORE_KERNEL_H2O_RELEASE: return "h2o_release";
    case ADORE_KERNEL_H2O_CHOICE: return "h2o_choice";
    case ADORE_KERNEL_H2O_PLACE: return "h2o_place";
    default: return "?";
  }
}

const char *adore_strerror(int code) {
  switch (code) {
    case ADORE_OK: return "ok";
    case ADORE_E_INVALID: return "invalid argument (null pointer, bad shape or value)";
    case ADORE_E_STATE: return "call out of order for this step, or step past max_positions";
    case ADORE_E_UNSUPPORTED:
      return "unsupported configuration (need head_dim in {64,128}, cache_slots <= 1024 or "
             "cache_slots - rebuild_budget - 1 >= max_positions, hidden % 8 == 0, max_positions <= 262144, "
             "ctrl_hidden <= 1024, ctrl_hidden % 4 == 0 in rescore mode; H2O mode: one layer, heads <= 255, "
             "max_positions <= about 7000, no rotary embedding, no forward; set_state in static mode only)";
    case ADORE_E_WORKSPACE: return "workspace too small or not 256-byte aligned";
    case ADORE_E_HIP: return "HIP runtime call failed";
    default: return "unknown error";
  }
}

int adore_abi_version(void) { return ADORE_ABI_VERSION; }

}  // extern "C"
