// H2O(Rebuilt) score source (paper Sec. 3.1, baselines 6 and 7: H2O evicts the tokens that contribute least to the
// cumulative attention; the rebuilt variant rebuilds K/V states of evicted tokens on top of it).
//
//   score[b][h][i]  = sum over the steps at which head h held a row of token i of the probability the step's query
//                     gave that row; fp32, added in step order; an evicted token keeps its score
//   release         per (b,h) on the head's own scores; how many rows a head gives up it counts itself
//   rebuild choice  per sequence: candidates = tokens at least one head is missing, ranked by the fp32 sum of their
//                   scores over the heads (head 0 first), ties to the lower position; a head that still holds a
//                   chosen token keeps its row, the others take their lowest free slots in rank order
//
// The attention kernel leaves every slot's logit and the row's (maximum, sum) behind; the release kernel turns them
// into probabilities and adds them to the scores before it ranks.  Everything runs on the caller's stream, behind
// the step's attention (the scores depend on it) and ahead of the re-projection.
#include "select_device.h"

namespace adore {

namespace {

constexpr int kChoiceThreads = 512;
constexpr int kChoiceWaves = kChoiceThreads / 64;

__global__ void h2o_init_scores_kernel(float *score, const float *init, int rows, int S, int N_max) {
  const size_t i = size_t(blockIdx.x) * blockDim.x + threadIdx.x;
  if (i >= size_t(rows) * S) return;
  const size_t row = i / S, pos = i - row * S;
  score[row * N_max + pos] = init ? init[i] : 0.f;
}

template <int KPL>
__global__ __launch_bounds__(256) void h2o_release_kernel(const int32_t *__restrict__ slot_src, int32_t *__restrict__ slot_dst,
                                                          const int32_t *__restrict__ insert_slot, float *score,
                                                          const float *__restrict__ logit, const float *__restrict__ ml,
                                                          int32_t *__restrict__ free_list, int32_t *__restrict__ released_pos,
                                                          int32_t *__restrict__ map_out, int32_t *__restrict__ rel_out,
                                                          int rows, int K, int N_max, int n, int m, int R1) {
  __shared__ uint32_t s_hist[4][256];           // one radix histogram per wave
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;                      // whole wave leaves together
  const int lane = threadIdx.x & 63;
  const int s_ins = insert_slot[row];
  const int32_t *sp = slot_src + size_t(row) * K;
  float *sc = score + size_t(row) * N_max;
  const float M = ml[size_t(row) * 2], L = ml[size_t(row) * 2 + 1];
  // what this step's query gave every row the head holds; the current token starts its score here
#pragma unroll
  for (int j = 0; j < KPL; ++j) {
    const int k = j * 64 + lane;
    if (k >= K) continue;
    const int pos = k == s_ins ? n : sp[k];
    if (pos < 0) continue;
    const float p = exp2f(logit[size_t(row) * K + k] - M) / L;
    sc[pos] = pos == n ? p : sc[pos] + p;
  }
  // the lane that wrote a score is the lane that reads it back below (same slot, same lane)
  release_row<KPL>(row, s_ins, slot_src, slot_dst, sc, free_list, released_pos, map_out, rel_out, K, n, -1, R1, nullptr,
                   s_hist[threadIdx.x >> 6], nullptr, m);
}

struct H2OChoiceArgs {
  int32_t *slot_pos;           // [B][H][K] after the release
  const float *score;          // [B][H][N_max]
  int32_t *free_list;          // [B][H][R1] in: ascending free slots; out: entry rho = the slot head h gives rank rho, -1 = it holds the token
  int32_t *rebuilt_pos;        // [B][Rdim]
  int32_t *insert_slot;        // [B][H]
  int32_t *map_out, *rb_out;   // the caller's copies, or null
  int K, H, N_max, n, R, R1, Rdim;
};

// One workgroup per sequence.  LDS: keys of tokens 0 .. n, how many heads hold each token (8 bits each), the select's
// scratch.  Writes the chosen positions (best first, then -1); h2o_place_kernel gives them their slots.
template <int KPL>
__global__ __launch_bounds__(kChoiceThreads) void h2o_choice_kernel(const H2OChoiceArgs a) {
  extern __shared__ uint64_t smem64[];
  const int n1 = a.n + 1, Rr = max(a.R, 1);
  uint64_t *s_all = smem64;                                     // [n + 1] ranking keys, 0 = every head holds the token
  uint64_t *s_keys = s_all + n1;                                // [Rr]
  uint64_t *s_ctl = s_keys + Rr;                                // [4]
  uint32_t *s_hist = reinterpret_cast<uint32_t *>(s_ctl + 4);   // [256]
  uint32_t *s_cnt = s_hist + 256;                               // [(n + 4) / 4] four counters per word
  int *s_sel = reinterpret_cast<int *>(s_cnt + (a.n + 4) / 4);  // [Rr] chosen positions, best first
  int *s_misc = s_sel + Rr;                                     // [0] collect's counter, [1] candidates
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

  for (int wd = tid; wd < (a.n + 4) / 4; wd += kChoiceThreads) s_cnt[wd] = 0;
  if (tid == 0) s_misc[1] = 0;
  __syncthreads();
  const int32_t *maps = a.slot_pos + size_t(b) * a.H * a.K;
  for (int idx0 = tid; idx0 < a.H * a.K; idx0 += 8 * kChoiceThreads) {   // eight loads on their way at a time
    int p[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int idx = idx0 + u * kChoiceThreads;
      p[u] = idx < a.H * a.K ? maps[idx] : -1;
    }
#pragma unroll
    for (int u = 0; u < 8; ++u)
      if (p[u] >= 0) atomicAdd(&s_cnt[p[u] >> 2], 1u << (8 * (p[u] & 3)));
  }
  __syncthreads();
  const float *sc = a.score + size_t(b) * a.H * a.N_max;
  int mine = 0;
  for (int i = tid; i < n1; i += kChoiceThreads) {
    // fp32, heads in order (the order is part of the result); the loads go out 32 (or eight) at a time: one after
    // the other they cost a trip to the L2 per head
    float agg = 0.f;
    int h = 0;
    for (; h + 32 <= a.H; h += 32) {
      float v[32];
#pragma unroll
      for (int u = 0; u < 32; ++u) v[u] = sc[size_t(h + u) * a.N_max + i];
#pragma unroll
      for (int u = 0; u < 32; ++u) agg = agg + v[u];
    }
    for (; h + 8 <= a.H; h += 8) {
      float v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = sc[size_t(h + u) * a.N_max + i];
#pragma unroll
      for (int u = 0; u < 8; ++u) agg = agg + v[u];
    }
    for (; h < a.H; ++h) agg = agg + sc[size_t(h) * a.N_max + i];
    const int holders = int((s_cnt[i >> 2] >> (8 * (i & 3))) & 255u);
    const uint64_t key = holders == a.H ? uint64_t(0) : rank_key(agg, i);
    s_all[i] = key;
    mine += key != 0;
  }
  if (mine) atomicAdd(&s_misc[1], mine);
  __syncthreads();
  const int r = min(a.R, s_misc[1]);            // uniform over the workgroup
  if (r > 0) {
    auto key_c = [&](int i) -> uint64_t { return s_all[i]; };
    uint64_t thr;
    int shift;
    radix_select(key_c, n1, r, s_hist, s_ctl, &thr, &shift);
    collect_sorted(key_c, n1, r, thr, shift, s_keys, &s_misc[0], s_sel);
  }
  for (int t = tid; t < a.Rdim; t += kChoiceThreads) {
    const int p = t < r ? s_sel[t] : -1;
    a.rebuilt_pos[size_t(b) * a.Rdim + t] = p;
    if (a.rb_out) a.rb_out[size_t(b) * a.Rdim + t] = p;
  }
}

// Placement, one wave per (sequence, head): the wave holds the head's row; the chosen tokens the head is missing take
// its free slots, lowest first, in rank order.  (Inside the choice kernel the heads of a sequence queued behind its
// eight waves, four rounds of loads and a serial walk over the ranks each.)
template <int KPL>
__global__ __launch_bounds__(256) void h2o_place_kernel(const H2OChoiceArgs a, int rows) {
  extern __shared__ int s_place[];               // [4 waves][R1 free slots + Rdim chosen positions]
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + wave;
  if (row >= rows) return;                       // whole wave leaves together; no barrier below
  const int b = row / a.H;
  int *fr = s_place + wave * (a.R1 + a.Rdim), *sel = fr + a.R1;
  for (int t = lane; t < a.R1; t += 64) fr[t] = a.free_list[size_t(row) * a.R1 + t];
  for (int t = lane; t < a.Rdim; t += 64) sel[t] = a.rebuilt_pos[size_t(b) * a.Rdim + t];
  int pos[KPL];
#pragma unroll
  for (int j = 0; j < KPL; ++j) {
    const int k = j * 64 + lane;
    pos[j] = k < a.K ? a.slot_pos[size_t(row) * a.K + k] : -1;
  }
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");   // the wave's LDS stores before its LDS loads
  __builtin_amdgcn_wave_barrier();
  int taken = 0, rho = 0;
  for (; rho < a.R; ++rho) {
    const int t = sel[rho];
    if (t < 0) break;                            // the chosen positions come first, then -1 (uniform over the wave)
    bool found = false;
#pragma unroll
    for (int j = 0; j < KPL; ++j) found |= pos[j] == t;
    const bool held = __ballot(found) != 0;
    int slot = -1;
    if (!held) slot = fr[taken++];
    if (lane == 0) {
      a.free_list[size_t(row) * a.R1 + rho] = slot;
      if (slot >= 0) {
        a.slot_pos[size_t(row) * a.K + slot] = t;
        if (a.map_out) a.map_out[size_t(row) * a.K + slot] = t;
      }
    }
  }
  for (int q = rho + lane; q < a.R; q += 64) a.free_list[size_t(row) * a.R1 + q] = -1;
  if (lane == 0) a.insert_slot[row] = fr[taken];   // taken <= R: the list holds R + 1 free slots
}

}  // namespace

size_t h2o_choice_lds_bytes(const adore_config &c, int n) {
  const size_t Rr = size_t(c.rebuild_budget > 0 ? c.rebuild_budget : 1);
  return size_t(n + 1) * 8 + Rr * 8 + 4 * 8 + 256 * 4 + size_t((n + 4) / 4) * 4 + Rr * 4 + 16;
}

hipError_t launch_h2o_init_scores(adore_ctx *ctx, const float *score_init, int S) {
  const adore_config &c = ctx->cfg;
  const size_t total = size_t(c.batch) * c.heads * S;
  hipLaunchKernelGGL(h2o_init_scores_kernel, dim3(unsigned((total + 255) / 256)), dim3(256), 0, ctx->stream, ctx->score,
                     score_init, c.batch * c.heads, S, c.max_positions);
  return hipGetLastError();
}

hipError_t launch_h2o_release(adore_ctx *ctx, int src, int dst, int32_t *map_out, int32_t *rel_out) {
  const adore_config &c = ctx->cfg;
  const int rows = c.batch * c.heads;
  const dim3 grid((rows + 3) / 4), block(256);
  ScopedTimer t(ctx, ADORE_KERNEL_H2O_RELEASE, ctx->stream);
#define ADORE_H2O_RELEASE(KPL)                                                                                         \
  ADORE_LAUNCH(t, (h2o_release_kernel<KPL>), grid, block, 0, ctx->stream, ctx->slot_pos[src], ctx->slot_pos[dst],      \
               ctx->insert_slot[src], ctx->score, ctx->att_logit, ctx->att_ml, ctx->free_list[dst], ctx->released_pos, \
               map_out, rel_out, rows, c.cache_slots, c.max_positions, ctx->n, c.cache_slots - c.rebuild_budget - 1,   \
               c.rebuild_budget + 1)
  if (c.cache_slots <= 128) ADORE_H2O_RELEASE(2);
  else if (c.cache_slots <= 256) ADORE_H2O_RELEASE(4);
  else if (c.cache_slots <= 512) ADORE_H2O_RELEASE(8);
  else ADORE_H2O_RELEASE(16);
#undef ADORE_H2O_RELEASE
  return hipGetLastError();
}

hipError_t launch_h2o_choice(adore_ctx *ctx, int maps, int lists, int n, int32_t *map_out, int32_t *rb_out) {
  const adore_config &c = ctx->cfg;
  H2OChoiceArgs a;
  a.slot_pos = ctx->slot_pos[maps]; a.score = ctx->score; a.free_list = ctx->free_list[lists];
  a.rebuilt_pos = ctx->rebuilt_pos[lists]; a.insert_slot = ctx->insert_slot[maps];
  a.map_out = map_out; a.rb_out = rb_out;
  a.K = c.cache_slots; a.H = c.heads; a.N_max = c.max_positions; a.n = n; a.R = c.rebuild_budget;
  a.R1 = c.rebuild_budget + 1; a.Rdim = max(c.rebuild_budget, 1);
  const size_t smem = h2o_choice_lds_bytes(c, n);
  ScopedTimer t(ctx, ADORE_KERNEL_H2O_CHOICE, ctx->stream);
  const dim3 grid(c.batch), block(kChoiceThreads);
  if (c.cache_slots <= 128) ADORE_LAUNCH(t, (h2o_choice_kernel<2>), grid, block, smem, ctx->stream, a);
  else if (c.cache_slots <= 256) ADORE_LAUNCH(t, (h2o_choice_kernel<4>), grid, block, smem, ctx->stream, a);
  else if (c.cache_slots <= 512) ADORE_LAUNCH(t, (h2o_choice_kernel<8>), grid, block, smem, ctx->stream, a);
  else ADORE_LAUNCH(t, (h2o_choice_kernel<16>), grid, block, smem, ctx->stream, a);
  if (hipGetLastError() != hipSuccess) return hipErrorLaunchFailure;
  ScopedTimer tp(ctx, ADORE_KERNEL_H2O_PLACE, ctx->stream);
  const int rows = c.batch * c.heads;
  const dim3 pgrid((rows + 3) / 4), pblock(256);
  const size_t psmem = size_t(4) * (a.R1 + a.Rdim) * 4;
  if (c.cache_slots <= 128) ADORE_LAUNCH(tp, (h2o_place_kernel<2>), pgrid, pblock, psmem, ctx->stream, a, rows);
  else if (c.cache_slots <= 256) ADORE_LAUNCH(tp, (h2o_place_kernel<4>), pgrid, pblock, psmem, ctx->stream, a, rows);
  else if (c.cache_slots <= 512) ADORE_LAUNCH(tp, (h2o_place_kernel<8>), pgrid, pblock, psmem, ctx->stream, a, rows);
  else ADORE_LAUNCH(tp, (h2o_place_kernel<16>), pgrid, pblock, psmem, ctx->stream, a, rows);
  return hipGetLastError();
}

}  // namespace adore
