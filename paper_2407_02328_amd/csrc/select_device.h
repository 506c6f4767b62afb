// Device code of the two selections of a decode step, shared by the stand-alone selection kernels and by the
// attention launch that carries them as extra workgroups.
//
// Ranking uses the 64-bit integer key of device_utils.h, so every selection has exactly one answer and is
// reproducible bit for bit.  Release is a wave-level binary radix select over the K keys of a row held in
// registers (K <= 1024).  The per-sequence choice is a most-significant-digit radix select over up to N_max
// keys with 8-bit digits and an LDS histogram; it stops as soon as the digit bucket holding the r-th key is
// taken whole.
#pragma once

#include "device_utils.h"

namespace adore {

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
// One wave per (b,h) row, no barriers; s_ins is the slot the attention of this step filled with token n;
// sc: the scores of the row's sequence by position (global memory or a copy in LDS);
// row_copy, if not null, receives the row as it stands after the release (K ints, e.g. in LDS);
// raw, if not null, holds what release_fetch read of the row earlier (so that the read is under way
// while something else is waited for).
// Lane L holds the keys of slots L, L+64, ...
// (KPL per lane).  The x lowest keys (x < 0: as many as leave m_keep rows) are found by a radix select, 8 bits a
// pass, with a histogram of the wave's own in LDS (hist: 256 words); digits on which all candidates agree are
// skipped.  Keys are distinct, so exactly x are taken.  (A bit-by-bit search with ballots, up to 64 passes of
// KPL ballots each, took 9 us of a 21 us chain next to the attention.)
// This lane's share of row `row` as it stands in memory: raw[j] = slot j*64 + lane (anything beyond K).
template <int KPL>
__device__ inline void release_fetch(int row, const int32_t *__restrict__ slot_src, int K, int (&raw)[KPL]) {
  const int lane = threadIdx.x & 63;
  const int32_t *sp = slot_src + size_t(row) * K;
#pragma unroll
  for (int j = 0; j < KPL; ++j) {
    const int k = j * 64 + lane;
    raw[j] = k < K ? sp[k] : -1;
  }
}

template <int KPL>
__device__ inline void release_row(int row, int s_ins, const int32_t *__restrict__ slot_src,
                                   int32_t *__restrict__ slot_dst, const float *sc,
                                   int32_t *__restrict__ free_list, int32_t *__restrict__ released_pos,
                                   int32_t *__restrict__ map_out, int32_t *__restrict__ rel_out, int K,
                                   int n, int x, int R1, int32_t *row_copy, uint32_t *hist, const int *raw = nullptr,
                                   int m_keep = 0) {
  const int lane = threadIdx.x & 63;
  const int32_t *sp = slot_src + size_t(row) * K;

  int pos[KPL];
  uint32_t khi[KPL], klo[KPL];
  uint32_t cand = 0;                            // bit j: slot j*64+lane holds a releasable token
  uint32_t or_hi = 0, or_lo = 0, and_hi = ~0u, and_lo = ~0u;
#pragma unroll
  for (int j = 0; j < KPL; ++j) {
    const int k = j * 64 + lane;
    pos[j] = k < K ? (k == s_ins ? n : (raw ? raw[j] : sp[k])) : -1;
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
  // x < 0: the row counts for itself how many rows it has to give up to be left with m_keep (the current token
  // included): heads that hold different numbers of rows (H2O mode) cannot be told from the host
  if (x < 0) need = max(0, nactive + 1 - m_keep);
  if (need > 0 && nactive > need) {
    // The `need` lowest keys are the `need` largest of the inverted keys: radix select on those, 8 bits a pass from
    // the top, the wave's own 256-bin histogram in LDS.  A pass is skipped when no two candidates differ in its
    // digit; the search ends as soon as the bin the rank falls into is taken whole (keys are distinct, so after
    // the last digit at the latest).
    bool done = false;
#pragma unroll 1
    for (int word = 1; word >= 0 && !done; --word) {
      const uint32_t diff = word ? diff_hi : diff_lo;
#pragma unroll 1
      for (int shift = 24; shift >= 0 && !done; shift -= 8) {
        if (((diff >> shift) & 0xffu) == 0u) continue;
        *reinterpret_cast<uint4 *>(hist + 4 * lane) = uint4{0u, 0u, 0u, 0u};
        wave_lds_fence();
#pragma unroll
        for (int j = 0; j < KPL; ++j) {
          const uint32_t kw = ~(word ? khi[j] : klo[j]);
          if ((active >> j) & 1u) atomicAdd(&hist[(kw >> shift) & 0xffu], 1u);
        }
        wave_lds_fence();
        int bin, rest, inbin;
        pick_bin(hist, lane, need, bin, rest, inbin);
        wave_lds_fence();                       // the reads above come before the next pass clears the bins
#pragma unroll
        for (int j = 0; j < KPL; ++j) {
          if (!((active >> j) & 1u)) continue;
          const int dgt = int(((~(word ? khi[j] : klo[j])) >> shift) & 0xffu);
          if (dgt > bin) sel |= 1u << j;        // above the bin: among the `need` largest for certain
          if (dgt != bin) active &= ~(1u << j);
        }
        need = rest;
        nactive = inbin;
        done = nactive == need;
      }
    }
  }
  if (need > 0) sel |= active;                  // what is left is exactly `need` keys

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
      if (row_copy) row_copy[k] = rel ? -1 : pos[j];
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

// The keys of tokens 0 .. n are kept in LDS for the passes of the per-sequence choice as long as they fit into
// 56 KB next to the residency bitmap; longer sequences recompute them from the scores in every pass.
__host__ __device__ inline bool choice_keys_cached(int n, int words) {
  return size_t(n + 1) * 8 + size_t(words) * 4 <= 56 * 1024;
}
// Beyond that a copy of the scores themselves (4 bytes a token, the key is made from it on the fly) still fits the
// LDS a workgroup may ask for (the stand-alone choice does; the limit leaves room for its other arrays): one read
// of the scores instead of one per pass up to about 33000 tokens.
constexpr size_t kChoiceLdsLimit = 152 * 1024;
__host__ __device__ inline bool choice_scores_cached(int n, int words) {
  return !choice_keys_cached(n, words) && size_t(n + 1) * 4 + size_t(words) * 4 + 16384 <= kChoiceLdsLimit;
}

// The choice for sequence b by one workgroup of any size.  res_row: the positions held by head 0 of the sequence
// after the release (uniform policy: every head of a sequence holds the same positions).  assign_heads: also
// enter the chosen positions into the slot maps of all heads and reserve the next free slot (otherwise whoever
// writes the rebuilt rows does that).  smem64: dynamic LDS of rebuild_choice_lds_bytes().
__device__ inline void rebuild_choice_block(const RebuildSelectArgs &a, int b, const int32_t *res_row,
                                            bool assign_heads, uint64_t *smem64) {
  const bool cached = choice_keys_cached(a.n, a.words);
  const bool sc_cached = choice_scores_cached(a.n, a.words);
  uint64_t *s_cache = smem64;                                   // [n + 1] keys, 0 = resident (if cached)
  float *s_score = reinterpret_cast<float *>(smem64);           // or [n + 1] scores (if sc_cached), padded to 8 bytes
  uint64_t *s_keys = smem64 + (cached ? a.n + 1 : sc_cached ? (a.n + 2) / 2 : 0);   // [max(r,1)]
  uint64_t *s_ctl = s_keys + max(a.r, 1);                       // [4]
  uint32_t *s_hist = reinterpret_cast<uint32_t *>(s_ctl + 4);   // [256]
  uint32_t *s_bits = s_hist + 256;                              // [words] residency bitmap
  int *s_sel = reinterpret_cast<int *>(s_bits + a.words);       // [max(r,1)] chosen positions, best first
  int *s_count = s_sel + max(a.r, 1);
  const int tid = threadIdx.x;
  const int r = a.r;

  if (r > 0) {
    for (int wd = tid; wd < a.words; wd += blockDim.x) s_bits[wd] = 0;
    __syncthreads();
    for (int k = tid; k < a.K; k += blockDim.x) {
      const int p = res_row[k];
      if (p >= 0) atomicOr(&s_bits[p >> 5], 1u << (p & 31));
    }
    __syncthreads();
    const float *sc = a.score + size_t(b) * a.N_max;
    auto key_of = [&](int i) -> uint64_t {
      return (s_bits[i >> 5] >> (i & 31)) & 1u ? uint64_t(0) : rank_key(sc[i], i);
    };
    uint64_t thr;
    int shift;
    if (cached) {   // one read of the scores instead of one per pass
      for (int i = tid; i <= a.n; i += blockDim.x) s_cache[i] = key_of(i);
      __syncthreads();
      auto key_c = [&](int i) -> uint64_t { return s_cache[i]; };
      radix_select(key_c, a.n + 1, r, s_hist, s_ctl, &thr, &shift);
      collect_sorted(key_c, a.n + 1, r, thr, shift, s_keys, s_count, s_sel);
    } else if (sc_cached) {   // the scores once, the keys from the copy in every pass
      for (int i = tid; i <= a.n; i += blockDim.x) s_score[i] = sc[i];
      __syncthreads();
      auto key_s = [&](int i) -> uint64_t {
        return (s_bits[i >> 5] >> (i & 31)) & 1u ? uint64_t(0) : rank_key(s_score[i], i);
      };
      radix_select(key_s, a.n + 1, r, s_hist, s_ctl, &thr, &shift);
      collect_sorted(key_s, a.n + 1, r, thr, shift, s_keys, s_count, s_sel);
    } else {
      radix_select(key_of, a.n + 1, r, s_hist, s_ctl, &thr, &shift);
      collect_sorted(key_of, a.n + 1, r, thr, shift, s_keys, s_count, s_sel);
    }
    for (int t = tid; t < r; t += blockDim.x) {
      a.rebuilt_pos[size_t(b) * a.Rdim + t] = s_sel[t];
      if (a.rb_out) a.rb_out[size_t(b) * a.Rdim + t] = s_sel[t];
    }
    if (assign_heads) {
      // rebuilt rank rho takes the rho-th lowest free slot of every head
      for (int idx = tid; idx < a.H * r; idx += blockDim.x) {
        const int h = idx / r, rho = idx - h * r;
        const int slot = a.free_list[(size_t(b) * a.H + h) * a.R1 + rho];
        a.slot_pos[(size_t(b) * a.H + h) * a.K + slot] = s_sel[rho];
        if (a.map_out) a.map_out[(size_t(b) * a.H + h) * a.K + slot] = s_sel[rho];
      }
    }
  }
  for (int t = r + tid; t < a.Rdim; t += blockDim.x) {
    a.rebuilt_pos[size_t(b) * a.Rdim + t] = -1;
    if (a.rb_out) a.rb_out[size_t(b) * a.Rdim + t] = -1;
  }
  if (assign_heads) {
    // the next free slot is reserved for the next token
    for (int h = tid; h < a.H; h += blockDim.x) {
      a.insert_slot[size_t(b) * a.H + h] = a.free_list[(size_t(b) * a.H + h) * a.R1 + r];
    }
  }
}

// The same choice in two parts, for a workgroup that finds out which positions head 0 keeps while it is
// already at work: choice_fill_keys needs only the scores (any subset of the workgroup's threads may run it, with
// their own tid / nthreads), choice_from_keys then drops the residents (res_row) and picks.  Requires
// choice_keys_cached(n, 0); LDS of ridden_choice_lds_bytes() at smem64.
__device__ inline void choice_fill_keys(const float *sc, int n, uint64_t *s_cache, int tid, int nthreads) {
  for (int i = tid; i <= n; i += nthreads) s_cache[i] = rank_key(sc[i], i);
}

__device__ inline void choice_from_keys(const RebuildSelectArgs &a, int b, const int32_t *res_row, uint64_t *smem64) {
  uint64_t *s_cache = smem64;                                   // [n + 1]
  uint64_t *s_keys = smem64 + a.n + 1;                          // [max(r,1)]
  uint64_t *s_ctl = s_keys + max(a.r, 1);                       // [4]
  uint32_t *s_hist = reinterpret_cast<uint32_t *>(s_ctl + 4);   // [256]
  int *s_sel = reinterpret_cast<int *>(s_hist + 256);           // [max(r,1)]
  int *s_count = s_sel + max(a.r, 1);
  const int tid = threadIdx.x;
  const int r = a.r;
  if (r > 0) {
    for (int k = tid; k < a.K; k += blockDim.x) {
      const int p = res_row[k];
      if (p >= 0) s_cache[p] = 0;                               // a resident is no candidate
    }
    __syncthreads();
    auto key_c = [&](int i) -> uint64_t { return s_cache[i]; };
    uint64_t thr;
    int shift;
    radix_select(key_c, a.n + 1, r, s_hist, s_ctl, &thr, &shift);
    collect_sorted(key_c, a.n + 1, r, thr, shift, s_keys, s_count, s_sel);
    for (int t = tid; t < r; t += blockDim.x) {
      a.rebuilt_pos[size_t(b) * a.Rdim + t] = s_sel[t];
      if (a.rb_out) a.rb_out[size_t(b) * a.Rdim + t] = s_sel[t];
    }
  }
  for (int t = r + tid; t < a.Rdim; t += blockDim.x) {
    a.rebuilt_pos[size_t(b) * a.Rdim + t] = -1;
    if (a.rb_out) a.rb_out[size_t(b) * a.Rdim + t] = -1;
  }
}

inline size_t ridden_choice_lds_bytes(int r, int n) {
  const size_t rr = size_t(r > 0 ? r : 1);
  return size_t(n + 1) * 8 + rr * 8 + 4 * 8 + 256 * 4 + rr * 4 + 8;
}

// n: position of the current token (keys of tokens 0 .. n)
inline size_t rebuild_choice_lds_bytes(int r, int words, int n) {
  const size_t rr = size_t(r > 0 ? r : 1);
  const size_t cache = choice_keys_cached(n, words) ? size_t(n + 1) * 8
                       : choice_scores_cached(n, words) ? size_t((n + 2) / 2) * 8 : 0;
  return cache + rr * 8 + 4 * 8 + 256 * 4 + size_t(words) * 4 + rr * 4 + 8;
}

}  // namespace adore
