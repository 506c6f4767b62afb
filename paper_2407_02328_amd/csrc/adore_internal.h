// Internal declarations shared by the host API and the kernel launchers.
// Not part of the public ABI (that is include/adore.h).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <cstdint>
#include <vector>

#include "adore.h"

namespace adore {

// Storage element tags.  bf16 values travel as raw 16-bit patterns.
struct bf16_t {
  uint16_t bits;
};

constexpr int kMaxSplits = 16;        // attention partials per (b,h) row
constexpr int kMaxSlots = 1024;       // largest K of a cache that releases (a row's keys live in one wave's registers)
constexpr int kMaxPositions = 1 << 18; // residency bitmap of a sequence lives in LDS
constexpr int kPromptChunk = 512;     // tokens per GRU input-projection launch at init
constexpr int kMaxCtrlSplit = 16;     // D-slices of the GRU input projection
constexpr int kCtrlSplitTokens = 256; // the projection is only sliced for launches of at most this many tokens
constexpr int kRing = 8;              // copies of the per-step lists (slot map, reserved slot, free slots, rebuilt tokens)
constexpr int kSyncEvery = 4;         // the side stream waits for the caller's stream once in this many steps
static_assert(kSyncEvery + 3 <= kRing, "a list is rewritten kRing - 1 steps after its last reader; see adore_api.hip");

// Static LDS of the attention kernel with 4 waves (merge of the lane groups: at most 32 groups x 64 or 16 x 128
// floats, and two floats per group), rounded up: what its extra workgroups have to leave room for.
constexpr size_t kAttendStaticLds = 8704;

struct TimedLaunch {
  int kernel;
  hipEvent_t start, stop;
};

}  // namespace adore

struct adore_ctx {
  adore_config cfg;
  adore_weights w;
  hipStream_t stream;        // the caller's stream: attention and the rebuild GEMM
  hipStream_t side;          // the selections (in RESCORE mode the rescoring ahead of them); equals `stream` when overlap is off
  hipStream_t side2;         // the controller, off the selections' chain; equals `stream` when overlap is off
  hipEvent_t ev_ctrl;        // recorded behind the controller of a step (on whichever stream ran it)
  hipEvent_t ev_att;         // recorded on `stream` after the last attention of a step, once in kSyncEvery steps
  hipEvent_t ev_join;        // recorded on `side` after the selections of a step
  hipEvent_t ev_in;          // ordered inputs: recorded on `stream` at the top of a step, the side stream starts behind it
  bool ordered;              // the side stream reads a step's inputs behind everything enqueued on `stream` before the call
  bool overlap;              // two-stream mode requested
  bool side_ready;           // side stream and events exist (made on first GPU use)

  // --- workspace sections (device) ---
  // Arrays marked xR are rings of kRing copies indexed by `cur`: a step's attention reads [cur] while its
  // selections write [cur + 1], so the selections of step n+1 may run while the GEMM of step n still
  // reads the lists of step n, and the side stream may run a few steps ahead of the caller's stream.
  char *ws_base;                    // the caller's workspace
  std::vector<size_t> guard_off;    // debug layout: where the guard words sit in it (empty: none)
  bool guards_ready;                // ... and whether they have their pattern yet
  char *cache_k, *cache_v;   // [L][B][H][K][d] storage type
  int32_t *slot_pos[adore::kRing];     // xR [B][H][K]   position per slot, -1 = free
  float *score;              // [B][N_max]  sigma_i
  float *z;                  // [B][d']     GRU state
  int32_t *insert_slot[adore::kRing];  // xR [B][H]      slot reserved for the next token
  int32_t *free_list[adore::kRing];    // xR [B][H][R+1] ascending free slots after the release
  int32_t *released_pos;     // [B][H][R+1]
  int32_t *rebuilt_pos[adore::kRing];  // xR [B][max(R,1)]
  int32_t *init_res;         // [B][K]      residents chosen at init, ascending position
  float *att_part;           // [B*H][kMaxSplits][d+2]
  float *att_logit;          // H2O mode: [B*H][K] the step's logits in base 2, as the attention kernel scaled them
  float *att_ml;             // H2O mode: [B*H][2] their maximum and the sum of exp2(logit - maximum) over the row
  float *gi;                 // [ksplit][tokens][3d'] GRU input pre-activations, per D-slice
  float *zseq;               // [B][kPromptChunk][d'] GRU states of a prompt chunk, between its scan and its scoring
  float *cvec;               // rescore mode: [B][N_max][d']  W_1 (z_i + pos_b) + b_1 of every token
  float *avec;               // rescore mode: [d']  W_1 pos_w  (what one unit of distance adds)
  void *fwd_q, *fwd_o;       // rebuild forward: [B*(R+1)][H*d] query rows / attention outputs of the layer in flight
  void *fwd_x;               // rebuild forward: [B*(R+1)][D]   rows handed from layer to layer
  void *rope;                // rope_base > 0: [N_max][d/2] (cos, sin) of pos * base^(-2j/d), fp64
  float2 *rope_f;            // ... and the same rounded to fp32

  // --- host-side step state ---
  bool inited;
  bool forward;              // initialised for the rebuild forward (adore_forward_step), not for attend/schedule/rebuild
  int32_t r_pending;         // forward: tokens chosen by the previous step, rebuilt by the next
  // where the slot reserved for the next token of (b,h) is found: insert_slot[cur][b*H + h] (stride 1, offset 0)
  // after an init, a set_state or a step through the stand-alone selection kernels; after a step whose
  // selections rode in the attention launch it is the entry behind the rebuilt tokens' slots in
  // free_list[cur][(b*H + h) * (R+1) + r]
  int32_t ins_stride, ins_off;
  bool ins_from_list;
  bool ride;                 // decode_step lets the selections ride in the attention launch when it can
  bool ride_fits;            // ... and this configuration allows it (score mode, slots, LDS at the last step)
  bool rode;                 // the last step did
  int32_t cur;               // ring index valid for the next attention
  int32_t steps_done;        // steps since the last init / set_state
  int32_t n;                 // position of the current / next token
  int32_t occ;               // occupied slots per (b,h) between steps
  int32_t r_step;            // rebuilt tokens chosen by this step's schedule
  bool scheduled;
  std::vector<uint8_t> attended, rebuilt;
  int32_t n_attended, n_rebuilt;

  // --- launch shape ---
  int32_t nsplit, chunk;     // attention: splits per row and slots per split
  int32_t attend_waves;      // attention: waves per workgroup (4, 8 or 16)

  // --- timing ---
  bool timing;
  std::vector<adore::TimedLaunch> timed;
  std::vector<hipEvent_t> event_pool;
};

namespace adore {

inline size_t elem_size(const adore_config &c) { return c.dtype == ADORE_BF16 ? 2 : 4; }

// The array that holds the reserved slots of ring copy `idx` (see adore_ctx::ins_stride).
inline const int32_t *reserved_slots(const adore_ctx *ctx, int idx) {
  return ctx->ins_from_list ? ctx->free_list[idx] : ctx->insert_slot[idx];
}

// Per-kernel timing.  When timing is on, the kernel is launched with hipExtLaunchKernelGGL, which ties
// the two events to the dispatch itself (its begin and end time stamps), so the elapsed time is the
// kernel's own duration without the queueing of an event bracket.
class ScopedTimer {
 public:
  ScopedTimer(adore_ctx *ctx, int kernel, hipStream_t stream);
  bool on() const { return on_; }
  hipEvent_t start() const { return ev_[0]; }
  hipEvent_t stop() const { return ev_[1]; }

 private:
  bool on_;
  hipEvent_t ev_[2];
};

#define ADORE_LAUNCH(TIMER, KERNEL, GRID, BLOCK, SMEM, STREAM, ...)                                   \
  do {                                                                                                \
    if ((TIMER).on())                                                                                 \
      hipExtLaunchKernelGGL(KERNEL, GRID, BLOCK, SMEM, STREAM, (TIMER).start(), (TIMER).stop(), 0,    \
                            __VA_ARGS__);                                                             \
    else                                                                                              \
      hipLaunchKernelGGL(KERNEL, GRID, BLOCK, SMEM, STREAM, __VA_ARGS__);                             \
  } while (0)

// Launchers.  Each validates nothing (the API did) and returns the launch status.  `st` is the
// stream to launch on; `src` / `dst` are indices into the rings of per-step lists.
// The selections of a step when they ride in the attention launch instead of running as kernels of their own.
struct RidingSelections {
  int dst;                 // ring copy they write
  int x, r;                // rows to release per (b,h), tokens to rebuild per sequence
  int32_t *map_out, *rel_out, *rb_out;   // the caller's copies, or null
};
// dynamic LDS of a workgroup that carries a sequence's selections in the attention launch at step n
size_t riding_lds_bytes(int n, int K, int r);
hipError_t launch_attend(adore_ctx *ctx, int layer, const void *q, const void *k_new,
                         const void *v_new, float *out, const RidingSelections *sel = nullptr);
hipError_t launch_ctrl_input(adore_ctx *ctx, hipStream_t st, const void *x, int ntok, int per_seq,
                             int seq_rows, int *ksplit_out);
hipError_t launch_ctrl_cell(adore_ctx *ctx, hipStream_t st, int nsteps, int pos0,
                            const float *score_override, int override_stride, int ksplit);
// The two selections also write the caller's copies of their results (slot map, released and rebuilt
// positions) when given a pointer, so a step needs no device-to-device copies.
hipError_t launch_release(adore_ctx *ctx, hipStream_t st, int src, int dst, int x, int32_t *map_out,
                          int32_t *rel_out);
hipError_t launch_rebuild_select(adore_ctx *ctx, hipStream_t st, int dst, int r, int32_t *map_out,
                                 int32_t *rb_out);
// map_dst / map_out: null, or the slot map (ring copy and the caller's) into which the kernel enters the rebuilt
// tokens' positions itself (when the per-sequence choice did not do it)
hipError_t launch_rebuild_gemm(adore_ctx *ctx, int layer, const void *hidden_layer, int lists, int r,
                               int32_t *map_dst = nullptr, int32_t *map_out = nullptr);
bool launch_plain_projection(adore_ctx *ctx, ScopedTimer &t, hipStream_t st, const void *x, const void *W, float *out,
                             int ntok, int per_seq, int seq_rows, int N, int D);
hipError_t launch_init_select(adore_ctx *ctx, int dst, int lists, int S, int keep, int r0);
hipError_t launch_init_copy(adore_ctx *ctx, const void *prompt_k, const void *prompt_v, int S,
                            int keep);
hipError_t launch_fill_i32(adore_ctx *ctx, int32_t *dst, int32_t value, size_t count);
// H2O mode (scores = attention collected per head; see csrc/h2o.hip).  All on the context's stream.
inline bool h2o_mode(const adore_ctx *ctx) { return ctx->cfg.score_mode == ADORE_SCORE_H2O; }
hipError_t launch_h2o_init_scores(adore_ctx *ctx, const float *score_init, int S);
hipError_t launch_h2o_init_select(adore_ctx *ctx, int dst, int lists, int S, int keep);
hipError_t launch_h2o_release(adore_ctx *ctx, int src, int dst, int32_t *map_out, int32_t *rel_out);
// n: the last position that exists (the current token of a step, S - 1 at init)
hipError_t launch_h2o_choice(adore_ctx *ctx, int maps, int lists, int n, int32_t *map_out, int32_t *rb_out);
size_t h2o_choice_lds_bytes(const adore_config &c, int n);
// rescore mode: the distance vector W_1 pos_w (once per init), and sigma of tokens 0..upto seen from token n
hipError_t launch_ctrl_avec(adore_ctx *ctx, hipStream_t st);
hipError_t launch_rescore(adore_ctx *ctx, hipStream_t st, int n, int upto);
// rebuild forward (one layer = qkv projection, attention of the r+1 rows, output projection with residual)
bool fwd_gemm_supported(const adore_config &c);
bool fwd_attend_mfma(const adore_config &c);
int fwd_attend_max_slots();
hipError_t launch_fwd_qkv(adore_ctx *ctx, int layer, const void *w_q_layer, const void *x_rows, bool by_position,
                          int r);
hipError_t launch_fwd_attend(adore_ctx *ctx, int layer, int r);
// rotary embedding (no-ops unless rope_base > 0): the angle table, once per init; the rotation of rows a projection
// wrote and did not rotate itself (the projections call it)
hipError_t launch_rope_table(adore_ctx *ctx);
hipError_t launch_rope_rows(adore_ctx *ctx, int layer, int lists, int r, int j0, int j1, bool queries, int cur_pos);
hipError_t launch_fwd_oproj(adore_ctx *ctx, const void *w_o_layer, const void *x_rows, bool by_position, void *out,
                            int out_rps, int out_cur, int r);

}  // namespace adore
