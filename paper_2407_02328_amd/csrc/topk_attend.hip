// Top-K attention over a whole sequence (paper Sec. 2.1: computing the full weights of a query and keeping the
// highest is the ideal sparsity; Sec. 2.2, first strategy, and App. "Implementation Details": the backbone is
// fine-tuned with attention whose weights outside the top K are masked out).  Causal, per (sequence, head):
//
//   w[i][j] = q_i . k_j  (j <= i);   kept(i) = the top_k largest w[i][.], equal weights to the lower j
//   out_i   = sum_{j in kept(i)} softmax_j(w[i][j] / sqrt(d)) v_j
//
// One workgroup of 8 waves takes 16 consecutive queries of one (sequence, head) and the keys they can see:
//
//   A  logits^T = K . Q^T on the matrix cores (16x16x32 bf16; the key rows come from global memory straight into
//      the operand layout, Q from an LDS tile), written to LDS as fp32, one row per query, -inf beyond the
//      diagonal.  All the weights of a query have to exist before its K-th largest is known; 16 x 2048 fp32 is
//      what LDS holds, and at 1024 keys two workgroups fit a compute unit.
//   S  one wave per query row: the row's maximum and its K-th largest weight by a radix select on the
//      order-preserving integer image of the floats: four passes of 8 bits over the row held in registers, each
//      a 256-bin histogram in LDS (wave-private, LDS atomics) scanned from the top; the rank left over in the last
//      bin says how many of the weights equal to the K-th largest stay, and ballots in position order say up to
//      which position.  As soon as at most 64 weights share the bits decided so far (as a rule after two passes)
//      they are gathered one per lane and ranked directly, which gives the last key that stays at once.  (A bit-by-bit search with ballots, 32 counting passes, took 5.6 ms of 8.0 ms at 512 rows of
//      1024 tokens, K = 96, in blocks of 32 queries; the radix select 1.5 ms of 3.4 ms.)
//   B  P = exp2((w - max) / sqrt(d) . log2 e) for the kept weights straight from the LDS rows (the maximum is
//      known, so there is no running rescale), as two bf16 terms (16 significant bits), and O^T += V^T . P^T on
//      the matrix cores.  V^T comes from a transposed copy of V made by a pass of its own ([d][S], zero-padded),
//      so that 8 consecutive keys of one head dimension are 16 contiguous bytes: the operand layout again.
//   M  the eight waves (each took every eighth block of 32 keys) add their partial sums through LDS in a fixed
//      order, normalise, round once and store.
//
// Phase B reads the very numbers phase S selected on, so the mask is exact with respect to the kernel's own fp32
// weights; against an fp64 evaluation two weights closer than the fp32 accumulation error may swap at the cut.
#include <hip/hip_runtime.h>

#include <cmath>
#include <mutex>

#include "adore.h"
#include "device_utils.h"

namespace adore {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kWaves = 8;
constexpr int kMaxSeq = 2048;        // longest sequence whose logit rows (16 queries) fit LDS
constexpr int kMaxLongSeq = 32768;   // longest sequence taken at all (rows in the workspace)
constexpr int kLongGrid = 512;       // workgroups of a launch over such sequences (two per compute unit; a multiple of 8)

// V [rows][S][d] -> V^T [rows][d][Sp], keys S .. Sp-1 as zeros.  One workgroup per 32 keys of one row.
__global__ __launch_bounds__(256) void topk_vt_kernel(const bf16_t *V, bf16_t *Vt, int S, int Sp, int d) {
  __shared__ uint16_t tile[32 * (128 + 2)];
  const int str = d + 2;
  const int key0 = blockIdx.x * 32;
  const size_t row = blockIdx.y;
  const uint16_t *src = reinterpret_cast<const uint16_t *>(V) + row * S * d;
  uint16_t *dst = reinterpret_cast<uint16_t *>(Vt) + row * d * Sp;
  for (int idx = threadIdx.x; idx < 32 * d; idx += 256) {
    const int key = idx / d, col = idx - key * d;
    tile[key * str + col] = key0 + key < S ? src[size_t(key0 + key) * d + col] : uint16_t(0);
  }
  __syncthreads();
  for (int idx = threadIdx.x; idx < 32 * d; idx += 256) {
    const int col = idx >> 5, key = idx & 31;
    dst[size_t(col) * Sp + key0 + key] = tile[key * str + col];
  }
}

struct TopkArgs {
  const bf16_t *Q, *K;   // [rows][S][d]
  const bf16_t *Vt;      // [rows][d][Sp]
  bf16_t *O;             // [rows][S][d]
  int S, Sp, topk, lstr; // lstr: floats per logit row
  int rows;
  int tiles;             // query blocks of the whole launch
  float *rowbuf;         // long sequences: [workgroups in flight][16][lstr] logit rows in the workspace
  int region0;           // bytes of the first LDS region (logit rows, later the merge buffer)
  float scale_log2;      // log2(e) / sqrt(d)
};

// Order-preserving image of a weight: larger float <=> larger integer; -inf (beyond the diagonal) -> 0, below
// every finite weight.  Adding +0 first makes a negative zero a positive one, so equal weights have equal images.
__device__ inline uint32_t weight_key(float x) {
  if (x == -INFINITY) return 0u;
  const uint32_t b = __float_as_uint(x + 0.0f);
  return b ^ ((b >> 31) ? 0xffffffffu : 0x80000000u);
}

// NQB: blocks of 16 queries per workgroup; NKMAX: keys of a row a lane can hold (64 * NKMAX >= the keys of a row)
// One tile of the launch: the 16 * NQB queries of block L (see the mapping below).  slot: which piece of the row
// buffer in the workspace this workgroup owns (long sequences only).
template <int DH, int NQB, int NKMAX>
__device__ inline void topk_tile(const TopkArgs &a, const int L, const int slot) {
  constexpr int KT = DH / 32;          // matrix instructions along d per 16x16 logit block
  constexpr int MB = DH / 16;          // 16-wide blocks of the head dimension
  constexpr int FIN = MB < kWaves ? MB : kWaves;   // waves that finish and store
  constexpr int OWN = MB / FIN;        // blocks of the head dimension such a wave finishes
  constexpr int NQ16 = NQB * 16;
  constexpr int QSTR = DH * 2 + 16;    // bytes per Q row in LDS
  constexpr int LPR = DH / 8;          // 16-byte vectors per row
  constexpr int RPW = NQ16 / kWaves;   // query rows a wave selects for
  extern __shared__ __align__(16) unsigned char smem[];
  // the weights of the block's queries: [NQ16][lstr] fp32 in LDS (later the merge buffer), or, for sequences whose
  // rows LDS cannot hold, in the workgroup's own piece of the workspace (written and read by this workgroup only)
  constexpr bool LONG = NKMAX == 0;
  float *s_log = LONG ? a.rowbuf + size_t(slot) * NQ16 * a.lstr : reinterpret_cast<float *>(smem);
  unsigned char *s_q = smem + a.region0;                                 // [NQ16][QSTR]
  uint32_t *s_T = reinterpret_cast<uint32_t *>(s_q + NQ16 * QSTR);       // [NQ16] image of the K-th largest weight
  int32_t *s_tie = reinterpret_cast<int32_t *>(s_T + NQ16);              // [NQ16] equal weights kept up to here
  float *s_max = reinterpret_cast<float *>(s_tie + NQ16);                // [NQ16]
  float *s_l = s_max + NQ16;                                             // [kWaves][NQ16]
  uint32_t *s_hist = reinterpret_cast<uint32_t *>(s_l + kWaves * NQ16);  // [kWaves][256] radix histograms

  // Workgroup -> (row, query block).  Consecutive workgroups go to the 8 XCDs in turn, each with an L2 of its own:
  // all query blocks of a row are given to one XCD (workgroups L, L + 8, L + 16 ...), so that the row's K and V^T
  // come from memory once instead of once per XCD; within a row the blocks with the most keys start first.
  const int nq = (a.S + NQ16 - 1) / NQ16;
  const int full = a.rows / 8 * 8;             // rows that form whole groups of 8
  int row_, qi;
  if (L < full * nq) {
    const int slot = L >> 3;
    row_ = slot / nq * 8 + (L & 7);
    qi = slot - slot / nq * nq;
  } else {
    const int rest = L - full * nq;
    row_ = full + rest / nq;
    qi = rest - rest / nq * nq;
  }
  const int qblk = nq - 1 - qi;
  const size_t bh = size_t(row_);
  const int q0 = qblk * NQ16;
  const int nkeys = min(a.S, q0 + NQ16);    // keys a query of this block can see
  const int nb32 = (nkeys + 31) / 32;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int c = lane & 15, g = lane >> 4;
  const int lstr = a.lstr;

  const bf16_t *Qb = a.Q + bh * a.S * DH;
  const bf16_t *Kb = a.K + bh * a.S * DH;
  const bf16_t *Vtb = a.Vt + bh * DH * a.Sp;

  // ---- the query tile ----
  for (int idx = tid; idx < NQ16 * LPR; idx += 64 * kWaves) {
    const int row = idx / LPR, ch = idx - row * LPR;
    u32x4 v = u32x4{0u, 0u, 0u, 0u};
    if (q0 + row < a.S) v = *reinterpret_cast<const u32x4 *>(Qb + size_t(q0 + row) * DH + ch * 8);
    *reinterpret_cast<u32x4 *>(s_q + row * QSTR + ch * 16) = v;
  }
  int qpos[NQB];
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb) qpos[qb] = q0 + qb * 16 + c;
  __syncthreads();

  // ---- A: logits^T of every eighth block of 32 keys ----
  {
    u32x4 kf[2][KT];
#define LOAD_K(BASE)                                                                         \
  _Pragma("unroll") for (int sb = 0; sb < 2; ++sb) {                                         \
    const int key_ = min((BASE) + sb * 16 + c, a.S - 1);                                     \
    _Pragma("unroll") for (int t = 0; t < KT; ++t)                                           \
      kf[sb][t] = *reinterpret_cast<const u32x4 *>(Kb + size_t(key_) * DH + (t * 4 + g) * 8); \
  }
    if (wave < nb32) { LOAD_K(wave * 32) }
    for (int blk = wave; blk < nb32; blk += kWaves) {
      const int base = blk * 32;
      f32x4 s[2][NQB];
#pragma unroll
      for (int sb = 0; sb < 2; ++sb)
#pragma unroll
        for (int qb = 0; qb < NQB; ++qb) s[sb][qb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int qb = 0; qb < NQB; ++qb)
#pragma unroll
        for (int t = 0; t < KT; ++t) {
          const u32x4 qv = *reinterpret_cast<const u32x4 *>(s_q + (qb * 16 + c) * QSTR + (t * 4 + g) * 16);
#pragma unroll
          for (int sb = 0; sb < 2; ++sb)
            s[sb][qb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*reinterpret_cast<const bf16x8 *>(&kf[sb][t]),
                                                                *reinterpret_cast<const bf16x8 *>(&qv), s[sb][qb], 0, 0, 0);
        }
      if (blk + kWaves < nb32) { LOAD_K(base + kWaves * 32) }
      // a lane holds, for its query, keys base + sb*16 + g*4 + i
#pragma unroll
      for (int sb = 0; sb < 2; ++sb)
#pragma unroll
        for (int qb = 0; qb < NQB; ++qb) {
          f32x4 w;
#pragma unroll
          for (int i = 0; i < 4; ++i) w[i] = base + sb * 16 + g * 4 + i <= qpos[qb] ? s[sb][qb][i] : -INFINITY;
          *reinterpret_cast<f32x4 *>(s_log + (qb * 16 + c) * lstr + base + sb * 16 + g * 4) = w;
        }
    }
#undef LOAD_K
  }
  __syncthreads();

  // ---- S: per query row, the maximum, the K-th largest weight and the cut among its equals ----
  {
    const int tmax = (nb32 * 32 + 63) / 64;   // 64-key groups the rows of this block have
    for (int rr = 0; rr < RPW; ++rr) {
      const int row = wave * RPW + rr;
      const int p = q0 + row;
      uint32_t T = 0xffffffffu;               // rows beyond the sequence keep nothing
      int tie = -1;
      float mx = 0.f;
      if (LONG && p < a.S) {
        // The row stays in memory (it was written by this workgroup and comes from the L2): every pass reads it
        // again, 64 keys at a time.  Four passes always; then the cut among the equal weights in position order.
        const float *lrow = s_log + row * lstr;
        const int nkp = nb32 * 32;
        mx = -INFINITY;
        for (int j = lane; j < nkp; j += 64) mx = fmaxf(mx, lrow[j]);
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
        if (p + 1 <= a.topk) {
          T = 1u;
          tie = 0x7fffffff;
        } else {
          uint32_t *hist = s_hist + wave * 256;
          uint32_t prefix = 0u;
          int need = a.topk;
#pragma unroll 1
          for (int shift = 24; shift >= 0; shift -= 8) {
#pragma unroll
            for (int i = 0; i < 4; ++i) hist[lane + 64 * i] = 0u;
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
            const uint32_t himask = shift == 24 ? 0u : 0xffffffffu << (shift + 8);
            for (int j = lane; j < nkp; j += 64) {
              const uint32_t uj = weight_key(lrow[j]);
              if (uj != 0u && (uj & himask) == prefix) atomicAdd(&hist[(uj >> shift) & 255u], 1u);
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
            int bin, rest, inbin;
            pick_bin(hist, lane, need, bin, rest, inbin);
            need = rest;
            prefix |= uint32_t(bin) << shift;
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
          }
          T = prefix;
          for (int j0 = 0; j0 < nkp && tie < 0; j0 += 64) {     // nkp is a multiple of 32: guard the last half group
            const uint32_t uj = j0 + lane < nkp ? weight_key(lrow[j0 + lane]) : 0u;
            unsigned long long m = __builtin_amdgcn_ballot_w64(uj == T);
            const int cnt = __builtin_popcountll(m);
            if (need > cnt) {
              need -= cnt;
            } else {
              for (int i = 1; i < need; ++i) m &= m - 1;
              tie = __builtin_ctzll(m) + j0;
            }
          }
        }
      }
      if constexpr (!LONG) if (p < a.S) {
        const float *lrow = s_log + row * lstr;
        uint32_t u[NKMAX];
        mx = -INFINITY;
#pragma unroll
        for (int t = 0; t < NKMAX; ++t) {
          u[t] = 0u;
          if (t < tmax) {
            const int j = lane + 64 * t;
            const float x = j < nb32 * 32 ? lrow[j] : -INFINITY;
            mx = fmaxf(mx, x);
            u[t] = weight_key(x);
          }
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
        if (p + 1 <= a.topk) {
          T = 1u;                             // below the image of every finite weight: all visible keys stay
          tie = 0x7fffffff;
        } else {
          // radix select, 8 bits a pass from the top: `prefix` = the bits of the K-th largest image decided so
          // far, `need` = its rank among the images that share them (1 = the largest)
          uint32_t *hist = s_hist + wave * 256;
          uint32_t prefix = 0u;
          int need = a.topk;
#pragma unroll 1
          for (int shift = 24; shift >= 0; shift -= 8) {
#pragma unroll
            for (int i = 0; i < 4; ++i) hist[lane + 64 * i] = 0u;
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");   // one wave's LDS operations run in order
            __builtin_amdgcn_wave_barrier();
            const uint32_t himask = shift == 24 ? 0u : 0xffffffffu << (shift + 8);
#pragma unroll
            for (int t = 0; t < NKMAX; ++t)
              if (t < tmax && u[t] != 0u && (u[t] & himask) == prefix) atomicAdd(&hist[(u[t] >> shift) & 255u], 1u);
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
            int bin, rest, inbin;
            pick_bin(hist, lane, need, bin, rest, inbin);
            need = rest;
            prefix |= uint32_t(bin) << shift;
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");   // the reads above come before the next writes
            __builtin_amdgcn_wave_barrier();
            if (shift > 0 && inbin <= 64) {
              // Few images share the bits decided so far: rank them directly instead of two or three more passes.
              // They are gathered in position order (ballots), one per lane; the one with need-1 others before it
              // in the order (image descending, position ascending) is the last key that stays.
              const uint32_t decided = 0xffffffffu << shift;
              uint32_t *cand = hist;          // [64] images, [64] positions: the histogram is not needed any more
              int base = 0;
#pragma unroll
              for (int t = 0; t < NKMAX; ++t) {
                if (t < tmax) {
                  const bool member = u[t] != 0u && (u[t] & decided) == prefix;
                  const unsigned long long m = __builtin_amdgcn_ballot_w64(member);
                  if (m != 0ull) {
                    if (member) {
                      const int slot = base + int(__builtin_amdgcn_mbcnt_hi(uint32_t(m >> 32), __builtin_amdgcn_mbcnt_lo(uint32_t(m), 0u)));
                      cand[slot] = u[t];
                      cand[64 + slot] = uint32_t(lane + 64 * t);
                    }
                    base += __builtin_popcountll(m);
                  }
                }
              }
              __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
              __builtin_amdgcn_wave_barrier();
              const bool have = lane < base;
              const uint32_t ui = have ? cand[lane] : 0u;
              const int pi = have ? int(cand[64 + lane]) : 0;
              int before = 0;
              for (int j = 0; j < base; ++j) {
                const uint32_t uj = cand[j];
                const int pj = int(cand[64 + j]);
                before += (uj > ui || (uj == ui && pj < pi)) ? 1 : 0;
              }
              const int last = __builtin_ctzll(__builtin_amdgcn_ballot_w64(have && before == need - 1));
              prefix = __shfl(ui, last, 64);
              tie = __shfl(pi, last, 64);
              __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
              __builtin_amdgcn_wave_barrier();
              break;
            }
          }
          T = prefix;   // all 32 bits decided: `need` of the weights equal to it stay, the lowest positions first
#pragma unroll
          for (int t = 0; t < NKMAX; ++t) {
            if (t < tmax && tie < 0) {
              unsigned long long m = __builtin_amdgcn_ballot_w64(u[t] == T);
              const int cnt = __builtin_popcountll(m);
              if (need > cnt) {
                need -= cnt;
              } else {
                for (int i = 1; i < need; ++i) m &= m - 1;   // drop the need-1 lowest positions
                tie = __builtin_ctzll(m) + 64 * t;
              }
            }
          }
        }
      }
      if (lane == 0) {
        s_T[row] = T;
        s_tie[row] = tie;
        s_max[row] = mx;
      }
    }
  }
  __syncthreads();

  // ---- B: O^T += V^T . P^T over every eighth block of 32 keys ----
  uint32_t Tq[NQB];
  int tieq[NQB];
  float negmax[NQB], lsum[NQB];
  f32x4 o[MB][NQB];
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb) {
    Tq[qb] = s_T[qb * 16 + c];
    tieq[qb] = s_tie[qb * 16 + c];
    negmax[qb] = -s_max[qb * 16 + c] * a.scale_log2;
    lsum[qb] = 0.f;
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) o[mb][qb] = f32x4{0.f, 0.f, 0.f, 0.f};
  }
  for (int blk = wave; blk < nb32; blk += kWaves) {
    const int base = blk * 32;
    u32x4 vf[MB];   // V^T: head dimension mb*16 + c, keys base + 8g .. + 7
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) vf[mb] = *reinterpret_cast<const u32x4 *>(Vtb + size_t(mb * 16 + c) * a.Sp + base + 8 * g);
    u32x4 bhi[NQB], blo[NQB];
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) {
      const float *src = s_log + (qb * 16 + c) * lstr + base + 8 * g;
      const f32x4 x0 = *reinterpret_cast<const f32x4 *>(src), x1 = *reinterpret_cast<const f32x4 *>(src + 4);
      uint32_t hi[8], lo[8];
      float psum = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float x = e < 4 ? x0[e] : x1[e - 4];
        const uint32_t uk = weight_key(x);
        const bool keep = uk > Tq[qb] || (uk == Tq[qb] && base + 8 * g + e <= tieq[qb]);
        const float pe = keep ? __builtin_amdgcn_exp2f(fmaf(x, a.scale_log2, negmax[qb])) : 0.f;
        psum += pe;
        // two bf16 terms: the upper 16 bits, and the upper 16 bits of what is left (exact, >= 0)
        hi[e] = __float_as_uint(pe);
        lo[e] = __float_as_uint(pe - __uint_as_float(hi[e] & 0xffff0000u));
      }
      lsum[qb] += psum;
#define PACK_HI(A, B) __builtin_amdgcn_perm(B, A, 0x07060302u)   /* (A >> 16) | (B & 0xffff0000) */
      bhi[qb] = u32x4{PACK_HI(hi[0], hi[1]), PACK_HI(hi[2], hi[3]), PACK_HI(hi[4], hi[5]), PACK_HI(hi[6], hi[7])};
      blo[qb] = u32x4{PACK_HI(lo[0], lo[1]), PACK_HI(lo[2], lo[3]), PACK_HI(lo[4], lo[5]), PACK_HI(lo[6], lo[7])};
#undef PACK_HI
    }
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
      for (int qb = 0; qb < NQB; ++qb) {
        o[mb][qb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*reinterpret_cast<const bf16x8 *>(&vf[mb]),
                                                            *reinterpret_cast<const bf16x8 *>(&bhi[qb]), o[mb][qb], 0, 0, 0);
        o[mb][qb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*reinterpret_cast<const bf16x8 *>(&vf[mb]),
                                                            *reinterpret_cast<const bf16x8 *>(&blo[qb]), o[mb][qb], 0, 0, 0);
      }
  }

  // ---- M: add the four waves' partial results in wave order ----
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb) {
    float l = lsum[qb];
    l += __shfl_xor(l, 16, 64);
    l += __shfl_xor(l, 32, 64);
    if (g == 0) s_l[wave * NQ16 + qb * 16 + c] = l;
  }
  __syncthreads();   // every wave is done with the logit rows, which the merge buffer overlays
  f32x4 *s_mrg = reinterpret_cast<f32x4 *>(smem);   // [kWaves][MB][NQB][64 lanes]
#pragma unroll
  for (int mb = 0; mb < MB; ++mb)
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) s_mrg[((wave * MB + mb) * NQB + qb) * 64 + lane] = o[mb][qb];
  __syncthreads();
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb) {
    const int q = q0 + qb * 16 + c;
    float L = 0.f;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) L += s_l[w * NQ16 + qb * 16 + c];
    const float inv = L > 0.f ? 1.f / L : 0.f;
#pragma unroll
    for (int j = 0; j < OWN; ++j) {
      if (wave >= FIN) break;
      const int mb = wave * OWN + j;
      f32x4 fin = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int w = 0; w < kWaves; ++w) {
        const f32x4 v = s_mrg[((w * MB + mb) * NQB + qb) * 64 + lane];
#pragma unroll
        for (int i = 0; i < 4; ++i) fin[i] += v[i];
      }
      if (q < a.S) {   // a lane holds 4 consecutive head dimensions of one query
        uint32_t r[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) r[i] = f32_to_bf16_rne(fin[i] * inv);
        *reinterpret_cast<u32x2 *>(a.O + (bh * a.S + q) * DH + mb * 16 + g * 4) = u32x2{r[0] | (r[1] << 16), r[2] | (r[3] << 16)};
      }
    }
  }
}

// Sequences whose logit rows live in LDS: one workgroup per tile.  Longer ones (NKMAX == 0): a grid of as many
// workgroups as the chip holds at once, each walking over tiles L, L + gridDim, ... with one piece of the row buffer
// of its own, so that the buffer is sized by the workgroups in flight, not by the tiles (rows * seq * seq floats).
// gridDim is a multiple of 8 there, so a workgroup's tiles stay on its XCD's rows.
template <int DH, int NQB, int NKMAX>
__global__ __launch_bounds__(64 * kWaves, NQB == 1 && NKMAX <= 16 ? 2 : 1) void topk_attend_kernel(const TopkArgs a) {
  if constexpr (NKMAX != 0) {
    topk_tile<DH, NQB, NKMAX>(a, blockIdx.x, 0);
  } else {
    for (int L = blockIdx.x; L < a.tiles; L += gridDim.x) {
      topk_tile<DH, NQB, NKMAX>(a, L, blockIdx.x);
      __syncthreads();   // the next tile reuses LDS and the workgroup's rows in the workspace
    }
  }
}

size_t padded_keys(int S) { return size_t(S + 31) / 32 * 32; }
size_t vt_bytes(int rows, int S, int d) { return (size_t(rows) * d * padded_keys(S) * 2 + 255) / 256 * 256; }

template <int DH, int NQB, int NKMAX>
hipError_t launch(const TopkArgs &base, int rows, hipStream_t st) {
  TopkArgs a = base;
  constexpr int NQ16 = NQB * 16;
  a.lstr = a.Sp + 4;
  const int logit_bytes = NKMAX == 0 ? 0 : NQ16 * a.lstr * 4;
  const int merge_bytes = kWaves * (DH / 16) * NQB * 64 * 16;
  a.region0 = (logit_bytes > merge_bytes ? logit_bytes : merge_bytes);
  const int lds = a.region0 + NQ16 * (DH * 2 + 16) + NQ16 * 12 + kWaves * NQ16 * 4 + kWaves * 256 * 4;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&topk_attend_kernel<DH, NQB, NKMAX>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, lds);
  if (e != hipSuccess) return e;
  a.rows = rows;
  a.tiles = ((a.S + NQ16 - 1) / NQ16) * rows;
  const dim3 grid(unsigned(NKMAX == 0 ? min(a.tiles, kLongGrid) : a.tiles)), block(64 * kWaves);
  hipLaunchKernelGGL((topk_attend_kernel<DH, NQB, NKMAX>), grid, block, lds, st, a);
  return hipGetLastError();
}

}  // namespace

}  // namespace adore

// ---- the entry point that allocates nothing ---------------------------------------------------------------
// The transposed copy of V of adore_topk_attention_static lives in this array instead of a caller's workspace.
// Every GPU the library runs on holds its own copy of it, at its own address, until the process ends.  In host
// code the name is only a handle for hipGetSymbolAddress: what kernels and copies get is the address looked up
// below, once per device.
static __device__ __align__(256) unsigned char scratch[ADORE_TOPK_STATIC_SCRATCH_BYTES];

namespace adore {
namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices] = {};   // by device ordinal; null = not looked up yet

// The address of `scratch` on the current device (looked up on the first call on that device), or null.
void *static_scratch() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void *ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
    g_scratch_ptr[dev] = ptr;
  }
  return g_scratch_ptr[dev];
}

// The launches of both entry points: the transposed copy of V into vt, then the attention.  seq <= kMaxSeq unless
// rowbuf is given.
int enqueue_topk(const void *q, const void *k, const void *v, void *out, void *vt, float *rowbuf, int rows, int seq,
                 int head_dim, int top_k, hipStream_t st) {
  const int Sp = int(padded_keys(seq));
  hipLaunchKernelGGL(topk_vt_kernel, dim3(Sp / 32, rows), dim3(256), 0, st, static_cast<const bf16_t *>(v),
                     static_cast<bf16_t *>(vt), seq, Sp, head_dim);
  if (hipGetLastError() != hipSuccess) return ADORE_E_HIP;
  TopkArgs a;
  a.Q = static_cast<const bf16_t *>(q);
  a.K = static_cast<const bf16_t *>(k);
  a.Vt = static_cast<const bf16_t *>(vt);
  a.O = static_cast<bf16_t *>(out);
  a.S = seq; a.Sp = Sp; a.topk = top_k; a.lstr = 0; a.region0 = 0; a.rows = rows;
  a.rowbuf = rowbuf;
  a.scale_log2 = 1.4426950408889634f / sqrtf(float(head_dim));
  hipError_t e;
  // 16 queries per workgroup: their fp32 weights take 64 KB of LDS at 1024 keys, so two workgroups (16 waves) share
  // a compute unit and hide each other's latencies (32 queries per workgroup, one workgroup per unit, read K and V
  // half as often and took 3.33 ms where this takes 2.27 ms)
  if (seq <= kMaxSeq / 2)
    e = head_dim == 128 ? launch<128, 1, 16>(a, rows, st) : launch<64, 1, 16>(a, rows, st);
  else if (seq <= kMaxSeq)
    e = head_dim == 128 ? launch<128, 1, 32>(a, rows, st) : launch<64, 1, 32>(a, rows, st);
  else   // logit rows in the workspace
    e = head_dim == 128 ? launch<128, 1, 0>(a, rows, st) : launch<64, 1, 0>(a, rows, st);
  return e == hipSuccess ? ADORE_OK : ADORE_E_HIP;
}

}  // namespace
}  // namespace adore

extern "C" {

size_t adore_topk_attention_workspace_bytes(int32_t rows, int32_t seq, int32_t head_dim) {
  if (rows <= 0 || seq <= 0 || head_dim <= 0) return 0;
  if (seq > adore::kMaxLongSeq || rows > 65535 || head_dim > 1024) return 0;   // nothing the entry point would take
  const size_t vt = adore::vt_bytes(rows, seq, head_dim);
  // sequences whose logit rows LDS cannot hold: 16 rows of fp32 weights per workgroup of 16 queries
  const size_t tiles = size_t(rows) * ((seq + 15) / 16);
  const size_t rowbuf = seq > adore::kMaxSeq ? (tiles < size_t(adore::kLongGrid) ? tiles : size_t(adore::kLongGrid)) * 16 *
                                                   (adore::padded_keys(seq) + 4) * 4
                                             : 0;
  return vt + (rowbuf + 255) / 256 * 256;
}

int adore_topk_attention(const void *q, const void *k, const void *v, void *out, void *workspace,
                         size_t workspace_bytes, int32_t rows, int32_t seq, int32_t head_dim, int32_t top_k,
                         void *hip_stream) {
  using namespace adore;
  if (!q || !k || !v || !out || !workspace || rows <= 0 || seq <= 0 || head_dim <= 0 || top_k < 1) return ADORE_E_INVALID;
  if ((head_dim != 64 && head_dim != 128) || seq > kMaxLongSeq || rows > 65535) return ADORE_E_UNSUPPORTED;
  if (workspace_bytes < adore_topk_attention_workspace_bytes(rows, seq, head_dim) ||
      (reinterpret_cast<uintptr_t>(workspace) & 255) != 0)
    return ADORE_E_WORKSPACE;
  float *rowbuf = reinterpret_cast<float *>(static_cast<char *>(workspace) + vt_bytes(rows, seq, head_dim));
  return enqueue_topk(q, k, v, out, workspace, rowbuf, rows, seq, head_dim, top_k, static_cast<hipStream_t>(hip_stream));
}

int adore_topk_attention_static(const void *q, const void *k, const void *v, void *out, int32_t rows, int32_t seq,
                                int32_t head_dim, int32_t top_k, void *hip_stream) {
  using namespace adore;
  if (!q || !k || !v || !out || rows <= 0 || seq <= 0 || head_dim <= 0 || top_k < 1) return ADORE_E_INVALID;
  if ((head_dim != 64 && head_dim != 128) || rows > 65535) return ADORE_E_UNSUPPORTED;
  // beyond kMaxSeq tokens the weights of the query blocks need a buffer of 512 x 16 rows of seq floats: not in this variant
  if (seq > kMaxSeq || vt_bytes(rows, seq, head_dim) > size_t(ADORE_TOPK_STATIC_SCRATCH_BYTES)) return ADORE_E_WORKSPACE;
  void *vt = static_scratch();
  if (!vt) return ADORE_E_HIP;
  return enqueue_topk(q, k, v, out, vt, nullptr, rows, seq, head_dim, top_k, static_cast<hipStream_t>(hip_stream));
}

}  // extern "C"
