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
#include "device_utils.h"

namespace adore {

namespace {

// Radix select.  key_of(i) for i in [0, ncand) returns the key of candidate i or 0
// if i is not a candidate.  Finds (*thr, *shift) such that exactly c candidates
// have (key >> shift) >= thr.  Needs 1 <= c <= number of candidates.
// s_hist: 256 uints; s_ctl: 4 uint64.  All threads of the block must call it.
template <class KeyFn>
__device__ inline void radix_select(KeyFn key_of, int ncand, int c, uint32_t *s_hist, uint64_t *s_ctl,
                                    uint64_t *thr, int *shift_out) {
  uint64_t prefix = 0;
  int remaining = c;
  int shift = 56;
  for (int pass = 0; pass < 8; ++pass, shift -= 8) {
    for (int t = threadIdx.x; t < 256; t += blockDim.x) s_hist[t] = 0;
    __syncthreads();
    for (int i = threadIdx.x; i < ncand; i += blockDim.x) {
      const uint64_t key = key_of(i);
      if (key != 0 && (pass == 0 || (key >> (shift + 8)) == prefix)) {
        atomicAdd(&s_hist[(key >> shift) & 0xff], 1u);
      }
    }
    __syncthreads();
    if (threadIdx.x < 64) {
      // lane L owns digits 4L..4L+3; suffix sums from the top digit down
      const int L = threadIdx.x;
      const uint32_t h0 = s_hist[4 * L], h1 = s_hist[4 * L + 1], h2 = s_hist[4 * L + 2], h3 = s_hist[4 * L + 3];
      const uint32_t own = h0 + h1 + h2 + h3;
      uint32_t incl = own;  // sum over lanes >= L
#pragma unroll
      for (int off = 1; off < 64; off <<= 1) {
        const uint32_t v = __shfl_down(incl, off, 64);
        if (L + off < 64) incl += v;
      }
      const uint32_t above_lane = incl - own;  // keys in digits of higher lanes
      // the lane where the running count first reaches `remaining`
      if (above_lane < uint32_t(remaining) && incl >= uint32_t(remaining)) {
        uint32_t above = above_lane;
        int digit;
        uint32_t cnt;
        if (above + h3 >= uint32_t(remaining)) { digit = 4 * L + 3; cnt = h3; }
        else if ((above += h3) + h2 >= uint32_t(remaining)) { digit = 4 * L + 2; cnt = h2; }
        else if ((above += h2) + h1 >= uint32_t(remaining)) { digit = 4 * L + 1; cnt = h1; }
        else { above += h1; digit = 4 * L; cnt = h0; }
        s_ctl[0] = uint64_t(digit);
        s_ctl[1] = uint64_t(uint32_t(remaining) - above);  // still to take inside this bucket
        s_ctl[2] = uint64_t(cnt);
      }
    }
    __syncthreads();
    prefix = (prefix << 8) | s_ctl[0];
    remaining = int(s_ctl[1]);
    const bool whole_bucket = s_ctl[2] == s_ctl[1];
    __syncthreads();
    if (whole_bucket) break;
  }
  if (shift < 0) shift = 0;  // all eight digits used: keys are distinct, the bucket held one key
  *thr = prefix;
  *shift_out = shift;
}

// Gathers the c selected keys (those with (key >> shift) >= thr) into s_keys in any
// order, then writes their positions best first to out_pos[0..c).  s_count: one int.
template <class KeyFn>
__device__ inline void collect_sorted(KeyFn key_of, int ncand, int c, uint64_t thr, int shift,
                                      uint64_t *s_keys, int *s_count, int32_t *out_pos) {
  if (threadIdx.x == 0) *s_count = 0;
  __syncthreads();
  for (int i = threadIdx.x; i < ncand; i += blockDim.x) {
    const uint64_t key = key_of(i);
    if (key != 0 && (key >> shift) >= thr) {
      const int idx = atomicAdd(s_count, 1);
      if (idx < c) s_keys[idx] = key;
    }
  }
  __syncthreads();
  for (int t = threadIdx.x; t < c; t += blockDim.x) {
    const uint64_t mine = s_keys[t];
    int rank = 0;
    for (int j = 0; j < c; ++j) rank += s_keys[j] > mine;
    out_pos[rank] = key_pos(mine);
  }
  __syncthreads();
}

// ---- release -------------------------------------------------------------------
// One wave per (b,h) row, no LDS, no barriers.  Lane L holds the keys of slots L, L+64, ...
// (KPL per lane).  The x lowest keys are found by a binary radix select from the top bit
// down: a ballot counts the candidates whose bit is 0; if there are at least `need` of them
// the ones drop out, otherwise all zeros are taken and the search goes on among the ones.
// Bits on which all candidates agree are skipped.  Keys are distinct, so exactly x are taken.
template <int KPL>
__global__ __launch_bounds__(256) void release_kernel(const int32_t *__restrict__ slot_src,
                                                      int32_t *__restrict__ slot_dst,
                                                      const int32_t *__restrict__ insert_slot,
                                                      const float *__restrict__ score,
                                                      int32_t *__restrict__ free_list,
                                                      int32_t *__restrict__ released_pos,
                                                      int32_t *__restrict__ map_out,
                                                      int32_t *__restrict__ rel_out, int rows, int K,
                                                      int H, int N_max, int n, int x, int R1) {
  __builtin_amdgcn_s_setprio(3);   // short, latency-bound work that shares compute units with the GEMM: its waves go first
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;                      // whole wave leaves together
  const int lane = threadIdx.x & 63;
  const int b = row / H;
  const int32_t *sp = slot_src + size_t(row) * K;
  const float *sc = score + size_t(b) * N_max;
  const int s_ins = insert_slot[row];           // the slot the attention of this step filled with token n

  int pos[KPL];
  uint32_t khi[KPL], klo[KPL];
  uint32_t cand = 0;                            // bit j: slot j*64+lane holds a releasable token
  uint32_t or_hi = 0, or_lo = 0, and_hi = ~0u, and_lo = ~0u;
#pragma unroll
  for (int j = 0; j < KPL; ++j) {
    const int k = j * 64 + lane;
    pos[j] = k < K ? (k == s_ins ? n : sp[k]) : -1;
  }
#pragma unroll
  for (int j = 0; j < KPL; ++j) {
    khi[j] = klo[j] = 0;
    if (pos[j] >= 0 && pos[j] != n) {
      const uint64_t key = rank_key(sc[pos[j]], pos[j]);
      khi[j] = uint32_t(key >> 32);
      klo[j] = uint32_t(key);
      cand |= 1u << j;
      or_hi |= khi[j]; or_lo |= klo[j];
      and_hi &= khi[j]; and_lo &= klo[j];
    }
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    or_hi |= __shfl_xor(or_hi, off, 64); or_lo |= __shfl_xor(or_lo, off, 64);
    and_hi &= __shfl_xor(and_hi, off, 64); and_lo &= __shfl_xor(and_lo, off, 64);
  }
  const uint32_t diff_hi = or_hi & ~and_hi, diff_lo = or_lo & ~and_lo;   // bits that tell candidates apart

  uint32_t active = cand, sel = 0;
  int need = x;
  int nactive = 0;                              // candidates still in play, whole row
#pragma unroll
  for (int j = 0; j < KPL; ++j) nactive += __popcll(__ballot((cand >> j) & 1u));
  if (need > 0) {
#pragma unroll 1
    for (int word = 1; word >= 0 && need > 0 && nactive > need; --word) {
      uint32_t diff = word ? diff_hi : diff_lo;
      while (diff != 0 && need > 0 && nactive > need) {
        const int bit = 31 - __clz(diff);
        diff &= ~(1u << bit);
        uint32_t zero = 0;                      // active candidates of this lane whose bit is 0
        int cnt0 = 0;
#pragma unroll
        for (int j = 0; j < KPL; ++j) {
          const uint32_t kw = word ? khi[j] : klo[j];
          const bool z = ((active >> j) & 1u) && !((kw >> bit) & 1u);
          zero |= uint32_t(z) << j;
          cnt0 += __popcll(__ballot(z));
        }
        if (cnt0 >= need) {
          active = zero;                        // the answer lies among the zeros
          nactive = cnt0;
        } else {
          sel |= zero;                          // all zeros are taken, go on among the ones
          active &= ~zero;
          need -= cnt0;
          nactive -= cnt0;
        }
      }
    }
    if (need > 0) sel |= active;                // what is left is exactly `need` keys
  }

  // ascending slot order = j major, lane minor
  int nfree = 0, nrel = 0;
  int32_t *dp = slot_dst + size_t(row) * K;
#pragma unroll
  for (int j = 0; j < KPL; ++j) {
    const int k = j * 64 + lane;
    const bool rel = (sel >> j) & 1u;
    const bool free_after = k < K && (pos[j] < 0 || rel);
    const uint64_t bf = __ballot(free_after), br = __ballot(rel);
    const uint64_t below = (uint64_t(1) << lane) - 1;
    if (free_after) {
      const int idx = nfree + __popcll(bf & below);
      if (idx < R1) free_list[size_t(row) * R1 + idx] = k;
    }
    if (rel) {
      const size_t at = size_t(row) * R1 + nrel + __popcll(br & below);
      released_pos[at] = pos[j];
      if (rel_out) rel_out[at] = pos[j];
    }
    if (k < K) {
      dp[k] = rel ? -1 : pos[j];
      if (map_out) map_out[size_t(row) * K + k] = rel ? -1 : pos[j];   // the caller's copy; rebuilt slots follow
    }
    nfree += __popcll(bf);
    nrel += __popcll(br);
  }
  for (int t = nrel + lane; t < R1; t += 64) {
    released_pos[size_t(row) * R1 + t] = -1;
    if (rel_out) rel_out[size_t(row) * R1 + t] = -1;
  }
}

// Release step of a row that gives nothing up (x = 0: the cache still has room for every token, which
// is always so when K - R - 1 >= N_max, the full-attention setting of Eq. 1).  Any K: the wave walks
// the row in chunks of 64 slots, enters the current token and lists the first R1 free slots.
__global__ __launch_bounds__(256) void release_none_kernel(const int32_t *__restrict__ slot_src,
                                                           int32_t *__restrict__ slot_dst,
                                                           const int32_t *__restrict__ insert_slot,
                                                           int32_t *__restrict__ free_list,
                                                           int32_t *__restrict__ released_pos,
                                                           int32_t *__restrict__ map_out,
                                                           int32_t *__restrict__ rel_out, int rows, int K, int n,
                                                           int R1) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;                      // whole wave leaves together
  const int lane = threadIdx.x & 63;
  const int32_t *sp = slot_src + size_t(row) * K;
  int32_t *dp = slot_dst + size_t(row) * K;
  const int s_ins = insert_slot[row];
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

// ---- per-sequence choice of the tokens to rebuild -------------------------------
struct RebuildSelectArgs {
  int32_t *slot_pos;           // [B][H][K]
  const float *score;          // [B][N_max]
  const int32_t *free_list;    // [B][H][R1]
  int32_t *rebuilt_pos;        // [B][Rdim]
  int32_t *insert_slot;        // [B][H]
  int32_t *map_out;            // [B][H][K] caller's slot map (already holds the map after the release), or null
  int32_t *rb_out;             // [B][Rdim] caller's copy of rebuilt_pos, or null
  int K, H, N_max, n, r, R1, Rdim, words;
};

__global__ __launch_bounds__(1024) void rebuild_select_kernel(const RebuildSelectArgs a) {
  __builtin_amdgcn_s_setprio(3);   // short, latency-bound work that shares compute units with the GEMM: its waves go first
  extern __shared__ uint64_t smem64[];
  uint64_t *s_keys = smem64;                                    // [max(r,1)]
  uint64_t *s_ctl = s_keys + max(a.r, 1);                       // [4]
  uint32_t *s_hist = reinterpret_cast<uint32_t *>(s_ctl + 4);   // [256]
  uint32_t *s_bits = s_hist + 256;                              // [words] residency bitmap
  int *s_sel = reinterpret_cast<int *>(s_bits + a.words);       // [max(r,1)] chosen positions, best first
  __shared__ int s_count;
  const int b = blockIdx.x;
  const int tid = threadIdx.x;
  const int r = a.r;

  if (r > 0) {
    for (int wd = tid; wd < a.words; wd += blockDim.x) s_bits[wd] = 0;
    __syncthreads();
    // uniform policy: every head of a sequence holds the same positions; head 0 is read
    const int32_t *sp0 = a.slot_pos + size_t(b) * a.H * a.K;
    for (int k = tid; k < a.K; k += blockDim.x) {
      const int p = sp0[k];
      if (p >= 0) atomicOr(&s_bits[p >> 5], 1u << (p & 31));
    }
    __syncthreads();
    const float *sc = a.score + size_t(b) * a.N_max;
    auto key_of = [&](int i) -> uint64_t {
      return (s_bits[i >> 5] >> (i & 31)) & 1u ? uint64_t(0) : rank_key(sc[i], i);
    };
    uint64_t thr;
    int shift;
    radix_select(key_of, a.n + 1, r, s_hist, s_ctl, &thr, &shift);
    collect_sorted(key_of, a.n + 1, r, thr, shift, s_keys, &s_count, s_sel);
    for (int t = tid; t < r; t += blockDim.x) {
      a.rebuilt_pos[size_t(b) * a.Rdim + t] = s_sel[t];
      if (a.rb_out) a.rb_out[size_t(b) * a.Rdim + t] = s_sel[t];
    }
    // rebuilt rank rho takes the rho-th lowest free slot of every head
    for (int idx = tid; idx < a.H * r; idx += blockDim.x) {
      const int h = idx / r, rho = idx - h * r;
      const int slot = a.free_list[(size_t(b) * a.H + h) * a.R1 + rho];
      a.slot_pos[(size_t(b) * a.H + h) * a.K + slot] = s_sel[rho];
      if (a.map_out) a.map_out[(size_t(b) * a.H + h) * a.K + slot] = s_sel[rho];
    }
  }
  for (int t = r + tid; t < a.Rdim; t += blockDim.x) {
    a.rebuilt_pos[size_t(b) * a.Rdim + t] = -1;
    if (a.rb_out) a.rb_out[size_t(b) * a.Rdim + t] = -1;
  }
  // the next free slot is reserved for the next token
  for (int h = tid; h < a.H; h += blockDim.x) {
    a.insert_slot[size_t(b) * a.H + h] = a.free_list[(size_t(b) * a.H + h) * a.R1 + r];
  }
}

// ---- init: residents and first rebuild set of a prompt ---------------------------
struct InitSelectArgs {
  int32_t *slot_pos;       // [B][H][K]
  const float *score;      // [B][N_max]
  int32_t *free_list;      // [B][H][R1]
  int32_t *rebuilt_pos;    // [B][Rdim]
  int32_t *insert_slot;    // [B][H]
  int32_t *init_res;       // [B][K]
  int K, H, N_max, S, keep, r0, R1, Rdim, words;
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
  const int b = blockIdx.x;
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
                                                        const int32_t *__restrict__ init_res, int B, int H,
                                                        int K, int S, int keep, int vec_per_row, size_t total) {
  const size_t i = size_t(blockIdx.x) * blockDim.x + threadIdx.x;
  if (i >= total) return;
  const int v = int(i % vec_per_row);
  size_t rest = i / vec_per_row;
  const int s = int(rest % keep);
  rest /= keep;                       // (l*B + b)*H + h
  const int b = int((rest / H) % B);
  const int pos = init_res[size_t(b) * K + s];
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
                 ctx->insert_slot[src], ctx->free_list[dst], ctx->released_pos, map_out, rel_out, rows,
                 c.cache_slots, ctx->n, c.rebuild_budget + 1);
    return hipGetLastError();
  }
#define ADORE_RELEASE(KPL)                                                                                   \
  ADORE_LAUNCH(t, (release_kernel<KPL>), grid, block, 0, st, ctx->slot_pos[src], ctx->slot_pos[dst],       \
                     ctx->insert_slot[src], ctx->score, ctx->free_list[dst], ctx->released_pos, map_out, rel_out, rows, \
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
  const size_t smem = size_t(max(r, 1)) * 8 + 4 * 8 + 256 * 4 + size_t(a.words) * 4 + size_t(max(r, 1)) * 4;
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
  const size_t smem = size_t(max(r0, 1)) * 8 + 4 * 8 + 256 * 4 + size_t(a.words) * 4 + size_t(max(r0, 1)) * 4;
  hipLaunchKernelGGL(init_select_kernel, dim3(c.batch), dim3(1024), smem, ctx->stream, a);
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
                     ctx->init_res, c.batch, c.heads, c.cache_slots, S, keep, vec_per_row, total);
  return hipGetLastError();
}

hipError_t launch_fill_i32(adore_ctx *ctx, int32_t *dst, int32_t value, size_t count) {
  const unsigned blocks = unsigned((count + 255) / 256);
  hipLaunchKernelGGL(fill_i32_kernel, dim3(blocks), dim3(256), 0, ctx->stream, dst, value, count);
  return hipGetLastError();
}

}  // namespace adore
