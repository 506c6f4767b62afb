// Stage 3: the two selections of a decode step, and their one-shot form at init.
//
//   release         per (b,h): free the x lowest-ranked occupied slots, never the
//                   current token's  (paper Sec. 2.2: discard the lowest sigma_i,
//                   remove an "older" state)
//   rebuild select  per sequence: the best r tokens that hold no cache row
//                   (paper Sec. 2.3: top-R sigma among released tokens), then
//                   rank rho -> rho-th lowest free slot of every head
//
// Ranking uses the 64-bit integer key of device_utils.h, so every selection has
// exactly one answer and is reproducible bit for bit.  Release is a wave-level
// binary radix select over the K keys of a row held in registers (K <= 1024).  The
// per-sequence choice is a most-significant-digit radix select over up to N_max
// keys with 8-bit digits and an LDS histogram; it stops as soon as the digit
// bucket holding the r-th key is taken whole.
#include "select_device.h"

namespace adore {

namespace {

template <int KPL>
__global__ __launch_bounds__(256) void release_kernel(const int32_t *__restrict__ slot_src,
                                                      int32_t *__restrict__ slot_dst,
                                                      const int32_t *__restrict__ insert_slot, int ins_stride,
                                                      int ins_off, const float *__restrict__ score,
                                                      int32_t *__restrict__ free_list,
                                                      int32_t *__restrict__ released_pos,
                                                      int32_t *__restrict__ map_out,
                                                      int32_t *__restrict__ rel_out, int rows, int K,
                                                      int H, int N_max, int n, int x, int R1) {
  __builtin_amdgcn_s_setprio(3);   // short, latency-bound work that shares compute units with the GEMM: its waves go first
  __shared__ uint32_t s_hist[4][256];           // one radix histogram per wave
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;                      // whole wave leaves together
  release_row<KPL>(row, insert_slot[size_t(row) * ins_stride + ins_off], slot_src, slot_dst,
                   score + size_t(row / H) * N_max, free_list, released_pos, map_out, rel_out, K, n, x, R1, nullptr,
                   s_hist[threadIdx.x >> 6]);
}

// Release step of a row that gives nothing up (x = 0: the cache still has room for every token, which
// is always so when K - R - 1 >= N_max, the full-attention setting of Eq. 1).  Any K: the wave walks
// the row in chunks of 64 slots, enters the current token and lists the first R1 free slots.
__global__ __launch_bounds__(256) void release_none_kernel(const int32_t *__restrict__ slot_src,
                                                           int32_t *__restrict__ slot_dst,
                                                           const int32_t *__restrict__ insert_slot, int ins_stride,
                                                           int ins_off, int32_t *__restrict__ free_list,
                                                           int32_t *__restrict__ released_pos,
                                                           int32_t *__restrict__ map_out,
                                                           int32_t *__restrict__ rel_out, int rows, int K, int n,
                                                           int R1) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;                      // whole wave leaves together
  const int lane = threadIdx.x & 63;
  const int32_t *sp = slot_src + size_t(row) * K;
  int32_t *dp = slot_dst + size_t(row) * K;
  const int s_ins = insert_slot[size_t(row) * ins_stride + ins_off];
  int nfree = 0;
  for (int k0 = 0; k0 < K; k0 += 64) {          // uniform trip count: the ballots see all 64 lanes
    const int k = k0 + lane;
    const int pos = k < K ? (k == s_ins ? n : sp[k]) : 0;
    const bool is_free = k < K && pos < 0;
    const uint64_t bf = __ballot(is_free);
    if (is_free) {
      const int idx = nfree + __popcll(bf & ((uint64_t(1) << lane) - 1));
      if (idx < R1) free_list[size_t(row) * R1 + idx] = k;
    }
    if (k < K) {
      dp[k] = pos;
      if (map_out) map_out[size_t(row) * K + k] = pos;
    }
    nfree += __popcll(bf);
  }
  for (int t = lane; t < R1; t += 64) {
    released_pos[size_t(row) * R1 + t] = -1;
    if (rel_out) rel_out[size_t(row) * R1 + t] = -1;
  }
}

__global__ __launch_bounds__(1024) void rebuild_select_kernel(const RebuildSelectArgs a) {
  __builtin_amdgcn_s_setprio(3);   // short, latency-bound work that shares compute units with the GEMM: its waves go first
  extern __shared__ uint64_t smem64[];
  // uniform policy: every head of a sequence holds the same positions; head 0 is read
  rebuild_choice_block(a, blockIdx.x, a.slot_pos + size_t(blockIdx.x) * a.H * a.K, true, smem64);
}

// ---- init: residents and first rebuild set of a prompt ---------------------------
struct InitSelectArgs {
  int32_t *slot_pos;       // [B][H][K]
  const float *score;      // [B][N_max]
  int32_t *free_list;      // [B][H][R1]
  int32_t *rebuilt_pos;    // [B][Rdim]
  int32_t *insert_slot;    // [B][H]
  int32_t *init_res;       // [B][K]; per_head: [B][H][K]
  int K, H, N_max, S, keep, r0, R1, Rdim, words;
  int per_head;            // 1: one workgroup per (sequence, head) with a score row of its own (H2O mode); it picks
                           // the head's residents only: the first rebuild set is chosen by another kernel
};

__global__ __launch_bounds__(1024) void init_select_kernel(const InitSelectArgs a) {
  extern __shared__ uint64_t smem64[];
  uint64_t *s_keys = smem64;                                    // [max(r0,1)]
  uint64_t *s_ctl = s_keys + max(a.r0, 1);                      // [4]
  uint32_t *s_hist = reinterpret_cast<uint32_t *>(s_ctl + 4);   // [256]
  uint32_t *s_bits = s_hist + 256;                              // [words] members of the resident set
  int *s_sel = reinterpret_cast<int *>(s_bits + a.words);       // [max(r0,1)]
  __shared__ int s_count;
  __shared__ int s_cnt[16];
  __shared__ int s_carry;
  const int b = blockIdx.x;     // per_head: the row index b * H + h
  const int tid = threadIdx.x;
  const float *sc = a.score + size_t(b) * a.N_max;

  for (int wd = tid; wd < a.words; wd += blockDim.x) s_bits[wd] = 0;
  __syncthreads();
  // residents: token S-1 and the best keep-1 older tokens
  if (tid == 0) s_bits[(a.S - 1) >> 5] |= 1u << ((a.S - 1) & 31);
  if (a.keep > 1) {
    auto key_all = [&](int i) -> uint64_t { return rank_key(sc[i], i); };
    uint64_t thr;
    int shift;
    radix_select(key_all, a.S - 1, a.keep - 1, s_hist, s_ctl, &thr, &shift);
    for (int i = tid; i < a.S - 1; i += blockDim.x) {
      if ((key_all(i) >> shift) >= thr) atomicOr(&s_bits[i >> 5], 1u << (i & 31));
    }
  }
  __syncthreads();
  // ascending positions -> init_res[b][0..keep)
  if (tid == 0) s_carry = 0;
  __syncthreads();
  for (int w0 = 0; w0 < a.words; w0 += blockDim.x) {
    const int wd = w0 + tid;
    const uint32_t bits = wd < a.words ? s_bits[wd] : 0u;
    // exclusive prefix of popcounts over the block
    const int cnt = __popc(bits);
    const int lane = tid & 63, wave = tid >> 6, nwaves = blockDim.x >> 6;
    int incl = cnt;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const int v = __shfl_up(incl, off, 64);
      if (lane >= off) incl += v;
    }
    if (lane == 63) s_cnt[wave] = incl;
    __syncthreads();
    int before = s_carry;
    for (int wv = 0; wv < wave; ++wv) before += s_cnt[wv];
    int idx = before + incl - cnt;
    uint32_t rest = bits;
    while (rest) {
      const int bit = __ffs(rest) - 1;
      rest &= rest - 1;
      a.init_res[size_t(b) * a.K + idx++] = wd * 32 + bit;
    }
    __syncthreads();
    if (tid == 0) {
      int all = 0;
      for (int wv = 0; wv < nwaves; ++wv) all += s_cnt[wv];
      s_carry += all;
    }
    __syncthreads();
  }
  if (a.per_head) {   // this head's slot map and its free slots in ascending order; the rest follows in h2o_choice_kernel
    const int32_t *res = a.init_res + size_t(b) * a.K;   // written above by this block
    for (int s = tid; s < a.K; s += blockDim.x) a.slot_pos[size_t(b) * a.K + s] = s < a.keep ? res[s] : -1;
    for (int idx = tid; idx < a.R1; idx += blockDim.x) a.free_list[size_t(b) * a.R1 + idx] = a.keep + idx;
    return;
  }
  // first rebuild set: best r0 of the non-residents
  if (a.r0 > 0) {
    auto key_pool = [&](int i) -> uint64_t {
      return (s_bits[i >> 5] >> (i & 31)) & 1u ? uint64_t(0) : rank_key(sc[i], i);
    };
    uint64_t thr;
    int shift;
    radix_select(key_pool, a.S, a.r0, s_hist, s_ctl, &thr, &shift);
    collect_sorted(key_pool, a.S, a.r0, thr, shift, s_keys, &s_count, s_sel);
  }
  for (int t = tid; t < a.Rdim; t += blockDim.x) {
    a.rebuilt_pos[size_t(b) * a.Rdim + t] = t < a.r0 ? s_sel[t] : -1;
  }
  // slot maps of every head: residents from slot 0, rebuilt next, the rest free
  const int32_t *res = a.init_res + size_t(b) * a.K;   // written above by this block
  for (int idx = tid; idx < a.H * a.K; idx += blockDim.x) {
    const int s = idx % a.K;
    int p = -1;
    if (s < a.keep) p = res[s];
    else if (s < a.keep + a.r0) p = s_sel[s - a.keep];
    a.slot_pos[size_t(b) * a.H * a.K + idx] = p;
  }
  for (int idx = tid; idx < a.H * a.R1; idx += blockDim.x) {
    a.free_list[size_t(b) * a.H * a.R1 + idx] = a.keep + idx % a.R1;
  }
  for (int h = tid; h < a.H; h += blockDim.x) a.insert_slot[size_t(b) * a.H + h] = a.keep + a.r0;
}

// cache[l][b][h][s][:] = prompt[l][b][h][init_res[b][s]][:] for s < keep, 16 bytes per thread
__global__ __launch_bounds__(256) void init_copy_kernel(const uint4 *__restrict__ prompt_k,
                                                        const uint4 *__restrict__ prompt_v,
                                                        uint4 *__restrict__ cache_k, uint4 *__restrict__ cache_v,
                                                        const int32_t *__restrict__ init_res, int res_heads, int B,
                                                        int H, int K, int S, int keep, int vec_per_row, size_t total) {
  const size_t i = size_t(blockIdx.x) * blockDim.x + threadIdx.x;
  if (i >= total) return;
  const int v = int(i % vec_per_row);
  size_t rest = i / vec_per_row;
  const int s = int(rest % keep);
  rest /= keep;                       // (l*B + b)*H + h
  const int b = int((rest / H) % B), h = int(rest % H);
  const int pos = init_res[(size_t(b) * res_heads + (res_heads > 1 ? h : 0)) * K + s];   // res_heads: 1, or H when heads differ
  const size_t src = (rest * S + pos) * vec_per_row + v;
  const size_t dst = (rest * K + s) * vec_per_row + v;
  cache_k[dst] = prompt_k[src];
  cache_v[dst] = prompt_v[src];
}

__global__ void fill_i32_kernel(int32_t *dst, int32_t value, size_t count) {
  const size_t i = size_t(blockIdx.x) * blockDim.x + threadIdx.x;
  if (i < count) dst[i] = value;
}

int round_up64(int v) { return (v + 63) / 64 * 64; }

}  // namespace

hipError_t launch_release(adore_ctx *ctx, hipStream_t st, int src, int dst, int x, int32_t *map_out,
                          int32_t *rel_out) {
  const adore_config &c = ctx->cfg;
  const int rows = c.batch * c.heads;
  const dim3 grid((rows + 3) / 4), block(256);
  ScopedTimer t(ctx, ADORE_KERNEL_RELEASE, st);
  if (c.cache_slots > kMaxSlots) {
    if (x != 0) return hipErrorInvalidValue;   // the API only admits such K when nothing is ever released
    ADORE_LAUNCH(t, release_none_kernel, grid, block, 0, st, ctx->slot_pos[src], ctx->slot_pos[dst],
                 reserved_slots(ctx, src), ctx->ins_stride, ctx->ins_off, ctx->free_list[dst], ctx->released_pos,
                 map_out, rel_out, rows, c.cache_slots, ctx->n, c.rebuild_budget + 1);
    return hipGetLastError();
  }
#define ADORE_RELEASE(KPL)                                                                                   \
  ADORE_LAUNCH(t, (release_kernel<KPL>), grid, block, 0, st, ctx->slot_pos[src], ctx->slot_pos[dst],       \
                     reserved_slots(ctx, src), ctx->ins_stride, ctx->ins_off, ctx->score, ctx->free_list[dst],     \
                     ctx->released_pos, map_out, rel_out, rows,                                                  \
                     c.cache_slots, c.heads, c.max_positions, ctx->n, x, c.rebuild_budget + 1)
  if (c.cache_slots <= 128) ADORE_RELEASE(2);
  else if (c.cache_slots <= 256) ADORE_RELEASE(4);
  else if (c.cache_slots <= 512) ADORE_RELEASE(8);
  else ADORE_RELEASE(16);
#undef ADORE_RELEASE
  return hipGetLastError();
}

hipError_t launch_rebuild_select(adore_ctx *ctx, hipStream_t st, int dst, int r, int32_t *map_out,
                                 int32_t *rb_out) {
  const adore_config &c = ctx->cfg;
  RebuildSelectArgs a;
  a.slot_pos = ctx->slot_pos[dst]; a.score = ctx->score; a.free_list = ctx->free_list[dst];
  a.rebuilt_pos = ctx->rebuilt_pos[dst]; a.insert_slot = ctx->insert_slot[dst];
  a.map_out = map_out; a.rb_out = rb_out;
  a.K = c.cache_slots; a.H = c.heads; a.N_max = c.max_positions; a.n = ctx->n; a.r = r;
  a.R1 = c.rebuild_budget + 1; a.Rdim = max(c.rebuild_budget, 1);
  a.words = (c.max_positions + 31) / 32;
  const size_t smem = rebuild_choice_lds_bytes(r, a.words, ctx->n);
  if (smem > 48 * 1024) {   // more than a workgroup gets without asking (host-side setting, once per process would do)
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&rebuild_select_kernel),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, int(kChoiceLdsLimit));
    if (e != hipSuccess) return e;
  }
  ScopedTimer t(ctx, ADORE_KERNEL_REBUILD_SELECT, st);
  ADORE_LAUNCH(t, rebuild_select_kernel, dim3(c.batch), dim3(1024), smem, st, a);
  return hipGetLastError();
}

hipError_t launch_init_select(adore_ctx *ctx, int dst, int lists, int S, int keep, int r0) {
  const adore_config &c = ctx->cfg;
  InitSelectArgs a;
  a.slot_pos = ctx->slot_pos[dst]; a.score = ctx->score; a.free_list = ctx->free_list[lists];
  a.rebuilt_pos = ctx->rebuilt_pos[lists]; a.insert_slot = ctx->insert_slot[dst]; a.init_res = ctx->init_res;
  a.K = c.cache_slots; a.H = c.heads; a.N_max = c.max_positions; a.S = S; a.keep = keep; a.r0 = r0;
  a.R1 = c.rebuild_budget + 1; a.Rdim = max(c.rebuild_budget, 1);
  a.words = (c.max_positions + 31) / 32;
  a.per_head = 0;
  const size_t smem = size_t(max(r0, 1)) * 8 + 4 * 8 + 256 * 4 + size_t(a.words) * 4 + size_t(max(r0, 1)) * 4;
  hipLaunchKernelGGL(init_select_kernel, dim3(c.batch), dim3(1024), smem, ctx->stream, a);
  return hipGetLastError();
}

// H2O mode: every head picks its residents on its own scores (slot map -> ring copy dst, ascending free slots ->
// ring copy lists, where h2o_choice_kernel takes them from).
hipError_t launch_h2o_init_select(adore_ctx *ctx, int dst, int lists, int S, int keep) {
  const adore_config &c = ctx->cfg;
  InitSelectArgs a;
  a.slot_pos = ctx->slot_pos[dst]; a.score = ctx->score; a.free_list = ctx->free_list[lists];
  a.rebuilt_pos = nullptr; a.insert_slot = nullptr; a.init_res = ctx->init_res;
  a.K = c.cache_slots; a.H = c.heads; a.N_max = c.max_positions; a.S = S; a.keep = keep; a.r0 = 0;
  a.R1 = c.rebuild_budget + 1; a.Rdim = max(c.rebuild_budget, 1);
  a.words = (c.max_positions + 31) / 32;
  a.per_head = 1;
  const size_t smem = 8 + 4 * 8 + 256 * 4 + size_t(a.words) * 4 + 4;
  hipLaunchKernelGGL(init_select_kernel, dim3(c.batch * c.heads), dim3(1024), smem, ctx->stream, a);
  return hipGetLastError();
}

hipError_t launch_init_copy(adore_ctx *ctx, const void *prompt_k, const void *prompt_v, int S, int keep) {
  const adore_config &c = ctx->cfg;
  const int vec_per_row = int(c.head_dim * elem_size(c) / 16);
  const size_t total = size_t(c.layers) * c.batch * c.heads * keep * vec_per_row;
  const unsigned blocks = unsigned((total + 255) / 256);
  hipLaunchKernelGGL(init_copy_kernel, dim3(blocks), dim3(256), 0, ctx->stream,
                     static_cast<const uint4 *>(prompt_k), static_cast<const uint4 *>(prompt_v),
                     reinterpret_cast<uint4 *>(ctx->cache_k), reinterpret_cast<uint4 *>(ctx->cache_v),
                     ctx->init_res, h2o_mode(ctx) ? c.heads : 1, c.batch, c.heads, c.cache_slots, S, keep, vec_per_row, total);
  return hipGetLastError();
}

hipError_t launch_fill_i32(adore_ctx *ctx, int32_t *dst, int32_t value, size_t count) {
  const unsigned blocks = unsigned((count + 255) / 256);
  hipLaunchKernelGGL(fill_i32_kernel, dim3(blocks), dim3(256), 0, ctx->stream, dst, value, count);
  return hipGetLastError();
}

}  // namespace adore
