// Rebuild forward, attention of one layer (paper Sec. 2.3 read in full): the r tokens chosen for
// rebuilding and the current token are all queries.  Every (sequence, head) has up to R+1 query
// rows over its K cache slots; a row at position p sees the slots whose position is <= p.
//
//   O[j][:] = sum_k softmax_k(Q[j] . Kc[k] / sqrt(d)) Vc[k]     over slots k with 0 <= pos[k] <= pos(j)
//
// Still memory-bound (the cache is streamed once for all rows: about R+1 flops per byte), but far
// too much arithmetic for the plain ALUs, so both products run on the matrix cores (16x16x32 bf16):
//
//   logits^T [slot][query] = Kc [slot][d] . Q^T     A = 16 cache rows, read from global memory straight
//                                                   into the operand layout (8 consecutive d per lane)
//   O^T [d][query]        += Vc^T [d][slot] . P^T   B = the probabilities exactly where the first product
//                                                   left them (a lane holds one query and 4+4 slots of
//                                                   two 16-slot blocks: that choice of 8 slots IS the
//                                                   k-order of the second product); A = V transposed
//                                                   through a wave-private LDS tile with the same k-order
//
// Probabilities enter the second product as two bf16 terms (upper 16 bits + the next 16 bits), so
// they carry 16 significant bits; sums are fp32; the output is rounded once to the storage type.
// One workgroup of 4 waves per (sequence, head); each wave streams a quarter of the slots with an
// online softmax (base 2), the four partial results are merged through LDS in a fixed order.
#include "device_utils.h"

namespace adore {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef int32_t i32x4 __attribute__((ext_vector_type(4)));

struct FwdAttendArgs {
  const bf16_t *Q;              // [B*nq][H*d]   query rows; row b*nq + j, j < r: rebuilt rank j, j == r: current token
  const bf16_t *Kc, *Vc;        // [B*H][K][d]   this layer's cache (the rows of the nq tokens already written)
  const int32_t *slot_pos;      // [B*H][K]      position per slot before this step's release; the current
                                //               token's slot is still marked free there
  const int32_t *insert_slot;   // [B*H]         the slot of the current token
  const int32_t *rebuilt_pos;   // [B][Rdim]     positions of the rebuilt tokens, by rank
  bf16_t *O;                    // [B*nq][H*d]
  int H, K, Kp, nq, r, Rdim, n, chunk;   // Kp = K rounded up to 4*chunk; chunk = slots per wave, multiple of 32
  float scale_log2;             // log2(e) / sqrt(d)
};

constexpr int kFwdWaves = 4;
constexpr float kNoMax = -1.0e30f;   // running maximum before anything has been seen (finite on purpose)
constexpr float kLazy = 8.f;         // the reference moves only when the maximum grows by more than 2^kLazy

template <int DH, int NQB>
constexpr int fwd_attend_lds_bytes(int Kp) {
  constexpr int q = NQB * 16 * (DH * 2 + 16);
  constexpr int ml = 2 * kFwdWaves * NQB * 16 * 4;
  constexpr int v = kFwdWaves * 32 * (DH * 2 + 8);
  constexpr int mrg = (DH / 16) * NQB * 64 * 16;
  return Kp * 4 + q + ml + (v > mrg ? v : mrg);
}

template <int DH, int NQB>
__global__ __launch_bounds__(256, (DH == 128 && NQB == 4) ? 1 : 2) void fwd_attend_kernel(const FwdAttendArgs a) {
  constexpr int KT = DH / 32;         // matrix instructions along d per 16x16 logit block
  constexpr int MB = DH / 16;         // 16-wide blocks of the head dimension
  constexpr int OWN = MB / kFwdWaves; // blocks of the head dimension a wave finishes and stores
  constexpr int VSTR = DH * 2 + 8;    // bytes per V row in LDS: 4 rows further = 32 bytes further in the banks
  constexpr int QSTR = DH * 2 + 16;   // bytes per Q row in LDS
  constexpr int LPR = DH / 8;         // lanes per cache row (16-byte loads)
  constexpr int RPI = 64 / LPR;       // cache rows per load instruction
  constexpr int NVL = 32 / RPI;       // V loads per lane and 32-slot block
  constexpr int NQ16 = NQB * 16;
  extern __shared__ __align__(16) unsigned char smem[];
  int32_t *s_pos = reinterpret_cast<int32_t *>(smem);                       // [Kp]
  unsigned char *s_q = smem + a.Kp * 4;                                     // [NQ16][QSTR]
  float *s_m = reinterpret_cast<float *>(s_q + NQ16 * QSTR);                // [4][NQ16]
  float *s_l = s_m + kFwdWaves * NQ16;                                      // [4][NQ16]
  unsigned char *s_big = reinterpret_cast<unsigned char *>(s_l + kFwdWaves * NQ16);

  const int bh = blockIdx.x;
  const int b = bh / a.H, h = bh - b * a.H;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int c = lane & 15, g = lane >> 4;
  const int Hd = a.H * DH;

  const bf16_t *Kb = a.Kc + size_t(bh) * a.K * DH;
  const bf16_t *Vb = a.Vc + size_t(bh) * a.K * DH;
  unsigned char *s_v = s_big + wave * 32 * VSTR;     // this wave's V tile [32][VSTR]
  const int vrow = lane / LPR, vch = lane - vrow * LPR;
  const int begin = wave * a.chunk;
  const int end = min(a.K, begin + a.chunk);
  u32x4 kf[2][KT], vr[NVL];
#define LOAD_K(BASE)                                                                        \
  _Pragma("unroll") for (int sb = 0; sb < 2; ++sb) {                                        \
    const int slot_ = min((BASE) + sb * 16 + c, a.K - 1);                                   \
    _Pragma("unroll") for (int t = 0; t < KT; ++t)                                          \
      kf[sb][t] = *reinterpret_cast<const u32x4 *>(Kb + size_t(slot_) * DH + (t * 4 + g) * 8); \
  }
#define LOAD_V(BASE)                                                                        \
  _Pragma("unroll") for (int it = 0; it < NVL; ++it) {                                      \
    const int slot_ = min((BASE) + it * RPI + vrow, a.K - 1);                               \
    vr[it] = *reinterpret_cast<const u32x4 *>(Vb + size_t(slot_) * DH + vch * 8);           \
  }

  // ---- every global read of the set-up is issued before any of them is waited for (a read of what the
  //      previous kernel wrote comes from memory, not from this XCD's cache: one round trip, not six) ----
  // positions of the slots (the current token's slot patched in), the query tile, the first cache block
  constexpr int QIT = (NQ16 * LPR + 255) / 256;      // query-tile vectors per thread
  constexpr int PIT = 4;                             // slot positions per thread and batch
  const int32_t *sp = a.slot_pos + size_t(bh) * a.K;
  const int s_ins = a.insert_slot[bh];
  u32x4 qv[QIT];
#pragma unroll
  for (int i = 0; i < QIT; ++i) {
    const int idx = tid + i * 256;
    const int row = idx / LPR, ch = idx - row * LPR;
    qv[i] = u32x4{0u, 0u, 0u, 0u};
    if (idx < NQ16 * LPR && row < a.nq)
      qv[i] = *reinterpret_cast<const u32x4 *>(a.Q + (size_t(b) * a.nq + row) * Hd + h * DH + ch * 8);
  }
  // position of this lane's query in every query block (padding rows: any value, their results are dropped).
  // A slot at position p is visible to a query at position P iff 0 <= p <= P: one unsigned comparison, a
  // free slot's -1 being the largest unsigned value.
  uint32_t qpos[NQB];
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb) {
    const int j = qb * 16 + c;
    qpos[qb] = uint32_t(j < a.r ? a.rebuilt_pos[size_t(b) * a.Rdim + j] : a.n);
  }
  int32_t pv[PIT];
#pragma unroll
  for (int i = 0; i < PIT; ++i) {
    const int k = tid + i * 256;
    pv[i] = k < a.K ? sp[k] : -1;
  }
  if (begin < end) {
    LOAD_K(begin)
    LOAD_V(begin)
  }
#pragma unroll
  for (int i = 0; i < PIT; ++i) {
    const int k = tid + i * 256;
    if (k < a.Kp) s_pos[k] = k == s_ins ? a.n : pv[i];
  }
  for (int k = tid + PIT * 256; k < a.Kp; k += 256) s_pos[k] = k < a.K ? (k == s_ins ? a.n : sp[k]) : -1;   // K > 1024
#pragma unroll
  for (int i = 0; i < QIT; ++i) {
    const int idx = tid + i * 256;
    const int row = idx / LPR, ch = idx - row * LPR;
    if (idx < NQ16 * LPR) *reinterpret_cast<u32x4 *>(s_q + row * QSTR + ch * 16) = qv[i];
  }
  __syncthreads();

  float m[NQB], lsum[NQB];
  f32x4 o[MB][NQB];
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb) {
    m[qb] = kNoMax;
    lsum[qb] = 0.f;
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) o[mb][qb] = f32x4{0.f, 0.f, 0.f, 0.f};
  }

  const float lazy_raw = kLazy / a.scale_log2;
  for (int base = begin; base < end; base += 32) {
    // ---- logits^T of 32 slots x all queries ----
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
    const bool more = base + 32 < end;
    if (more) { LOAD_K(base + 32) }

    // ---- V rows of the block into this wave's LDS tile; rows of free slots as zeros (a free slot may
    //      hold anything, and 0 x NaN would poison the product) ----
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");   // the previous block's reads of the tile come first
#pragma unroll
    for (int it = 0; it < NVL; ++it) {
      const int row = it * RPI + vrow;
      const bool ok = s_pos[base + row] >= 0;
      const u32x4 v = ok ? vr[it] : u32x4{0u, 0u, 0u, 0u};
      u32x2 *dst = reinterpret_cast<u32x2 *>(s_v + row * VSTR + vch * 16);
      dst[0] = u32x2{v.x, v.y};
      dst[1] = u32x2{v.z, v.w};
    }
    if (more) { LOAD_V(base + 32) }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();

    // ---- online softmax; the probabilities become the B operand of the second product ----
    // a lane holds, for its query, slots  base + g*4 + i  (sb = 0)  and  base + 16 + g*4 + i  (sb = 1).
    // The running maximum m (in units of the raw dot product) only moves when the block's maximum exceeds
    // it by more than kLazy / scale: until then probabilities are taken against the old reference (they
    // stay below 2^kLazy) and the accumulators need no rescaling.  m starts at a large negative finite
    // value, so that no case distinction for "nothing visible yet" is needed: exp2(-inf) = 0.
    i32x4 sp4[2];
#pragma unroll
    for (int sb = 0; sb < 2; ++sb) sp4[sb] = *reinterpret_cast<const i32x4 *>(s_pos + base + sb * 16 + g * 4);
    u32x4 bhi[NQB], blo[NQB];
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) {
      float x[8];
      float bm = -INFINITY;
#pragma unroll
      for (int sb = 0; sb < 2; ++sb)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          x[sb * 4 + i] = uint32_t(sp4[sb][i]) <= qpos[qb] ? s[sb][qb][i] : -INFINITY;
          bm = fmaxf(bm, x[sb * 4 + i]);
        }
      bm = fmaxf(bm, __shfl_xor(bm, 16, 64));
      bm = fmaxf(bm, __shfl_xor(bm, 32, 64));
      const bool move = bm > m[qb] + lazy_raw;          // the same in the four lanes of a query
      if (__builtin_amdgcn_ballot_w64(move) != 0) {
        const float alpha = move ? __builtin_amdgcn_exp2f((m[qb] - bm) * a.scale_log2) : 1.f;
        m[qb] = move ? bm : m[qb];
        lsum[qb] *= alpha;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
          for (int i = 0; i < 4; ++i) o[mb][qb][i] *= alpha;
      }
      const float neg_m = -m[qb] * a.scale_log2;
      float p[8], psum = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        p[e] = __builtin_amdgcn_exp2f(fmaf(x[e], a.scale_log2, neg_m));
        psum += p[e];
      }
      lsum[qb] += psum;
      // two bf16 terms per probability: the upper 16 bits, and the upper 16 bits of what is left (16
      // significant bits in all, rounded down); the upper halves of two floats are packed by one byte permute
      uint32_t hi[8], lo[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        hi[e] = __float_as_uint(p[e]);
        lo[e] = __float_as_uint(p[e] - __uint_as_float(hi[e] & 0xffff0000u));    // exact, >= 0
      }
#define PACK_HI(A, B) __builtin_amdgcn_perm(B, A, 0x07060302u)   /* (A >> 16) | (B & 0xffff0000) */
      bhi[qb] = u32x4{PACK_HI(hi[0], hi[1]), PACK_HI(hi[2], hi[3]), PACK_HI(hi[4], hi[5]), PACK_HI(hi[6], hi[7])};
      blo[qb] = u32x4{PACK_HI(lo[0], lo[1]), PACK_HI(lo[2], lo[3]), PACK_HI(lo[4], lo[5]), PACK_HI(lo[6], lo[7])};
#undef PACK_HI
    }

    // ---- O^T += V^T . P^T ----
    // the V^T fragment of the next 16 head dimensions is fetched from LDS before the matrix instructions of
    // the current ones; the two terms of a probability go to the same accumulator NQB instructions apart
    const uint16_t *vt = reinterpret_cast<const uint16_t *>(s_v);
#define VT_FRAG(DST, MBI)                                                                          \
  {                                                                                                \
    uint32_t w_[4];                                                                                \
    _Pragma("unroll") for (int e2 = 0; e2 < 4; ++e2) {                                             \
      const int slot0_ = (e2 < 2 ? 0 : 16) + g * 4 + (e2 & 1) * 2;   /* k-values 2*e2, 2*e2+1 */   \
      const uint32_t lo16_ = vt[(slot0_ * VSTR) / 2 + (MBI) * 16 + c];                             \
      const uint32_t hi16_ = vt[((slot0_ + 1) * VSTR) / 2 + (MBI) * 16 + c];                       \
      w_[e2] = lo16_ | (hi16_ << 16);                                                              \
    }                                                                                              \
    DST = u32x4{w_[0], w_[1], w_[2], w_[3]};                                                       \
  }
    u32x4 vf[2];
    VT_FRAG(vf[0], 0)
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
      if (mb + 1 < MB) { VT_FRAG(vf[(mb + 1) & 1], mb + 1) }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int qb = 0; qb < NQB; ++qb)
        o[mb][qb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*reinterpret_cast<const bf16x8 *>(&vf[mb & 1]),
                                                            *reinterpret_cast<const bf16x8 *>(&bhi[qb]), o[mb][qb], 0, 0, 0);
#pragma unroll
      for (int qb = 0; qb < NQB; ++qb)
        o[mb][qb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*reinterpret_cast<const bf16x8 *>(&vf[mb & 1]),
                                                            *reinterpret_cast<const bf16x8 *>(&blo[qb]), o[mb][qb], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
#undef VT_FRAG
  }
#undef LOAD_K
#undef LOAD_V

  // ---- merge the four waves: common maximum per query, then sums in wave order ----
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb) {
    float l = lsum[qb];
    l += __shfl_xor(l, 16, 64);
    l += __shfl_xor(l, 32, 64);
    lsum[qb] = l;
    if (g == 0) {
      s_m[wave * NQ16 + qb * 16 + c] = m[qb];
      s_l[wave * NQ16 + qb * 16 + c] = l;
    }
  }
  __syncthreads();   // also: every wave is done with its V tile, which the merge buffer overlays
  float inv_l[NQB];
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb) {
    float M = kNoMax;
#pragma unroll
    for (int w = 0; w < kFwdWaves; ++w) M = fmaxf(M, s_m[w * NQ16 + qb * 16 + c]);
    float L = 0.f, mine = 0.f;
#pragma unroll
    for (int w = 0; w < kFwdWaves; ++w) {
      const float f = __builtin_amdgcn_exp2f((s_m[w * NQ16 + qb * 16 + c] - M) * a.scale_log2);   // 0 for a wave that saw nothing
      L += f * s_l[w * NQ16 + qb * 16 + c];
      if (w == wave) mine = f;
    }
    inv_l[qb] = L > 0.f ? 1.f / L : 0.f;
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
      for (int i = 0; i < 4; ++i) o[mb][qb][i] *= mine;
  }
  // wave w finishes head-dimension blocks w*OWN .. w*OWN+OWN-1: in round t wave t lays out its whole
  // result, every wave adds its own blocks
  f32x4 *s_mrg = reinterpret_cast<f32x4 *>(s_big);   // [MB][NQB][64 lanes]
  f32x4 fin[OWN][NQB];
#pragma unroll
  for (int j = 0; j < OWN; ++j)
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) fin[j][qb] = f32x4{0.f, 0.f, 0.f, 0.f};
  for (int t = 0; t < kFwdWaves; ++t) {
    if (wave == t) {
#pragma unroll
      for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int qb = 0; qb < NQB; ++qb) s_mrg[(mb * NQB + qb) * 64 + lane] = o[mb][qb];
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < OWN; ++j)
#pragma unroll
      for (int qb = 0; qb < NQB; ++qb) {
        const f32x4 v = s_mrg[((wave * OWN + j) * NQB + qb) * 64 + lane];
#pragma unroll
        for (int i = 0; i < 4; ++i) fin[j][qb][i] += v[i];
      }
    __syncthreads();
  }
  // ---- normalise, round once, store: a lane holds 4 consecutive d of one query ----
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb) {
    const int j = qb * 16 + c;
    if (j < a.nq) {
      bf16_t *orow = a.O + (size_t(b) * a.nq + j) * Hd + h * DH;
#pragma unroll
      for (int jj = 0; jj < OWN; ++jj) {
        const int d0 = (wave * OWN + jj) * 16 + g * 4;
        uint32_t r[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) r[i] = f32_to_bf16_rne(fin[jj][qb][i] * inv_l[qb]);
        *reinterpret_cast<u32x2 *>(orow + d0) = u32x2{r[0] | (r[1] << 16), r[2] | (r[3] << 16)};
      }
    }
  }
}

template <int DH>
hipError_t launch_dh(adore_ctx *ctx, const FwdAttendArgs &a, int rows) {
  ScopedTimer t(ctx, ADORE_KERNEL_FWD_ATTEND, ctx->stream);
  const dim3 grid(rows), block(64 * kFwdWaves);
  const int nqb = (a.nq + 15) / 16;
#define FWD_CASE(N)                                                                                       \
  case N: {                                                                                               \
    const int lds = fwd_attend_lds_bytes<DH, N>(a.Kp);                                                    \
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&fwd_attend_kernel<DH, N>),          \
                                       hipFuncAttributeMaxDynamicSharedMemorySize, lds);                  \
    if (e != hipSuccess) return e;                                                                        \
    ADORE_LAUNCH(t, (fwd_attend_kernel<DH, N>), grid, block, lds, ctx->stream, a);                        \
    break;                                                                                                \
  }
  switch (nqb) {
    FWD_CASE(1)
    FWD_CASE(2)
    FWD_CASE(3)
    FWD_CASE(4)
    default: return hipErrorInvalidValue;
  }
#undef FWD_CASE
  return hipGetLastError();
}

// The same attention for storage types and shapes the kernel above does not take (fp32 storage, more than 64 rows per
// sequence): one wave per (sequence, head, query row), the definition written out.  Logits of the visible slots go to
// LDS (a lane takes every 64th slot and walks its key row), maximum and sum over the wave, then a lane takes every
// 64th element of the head dimension and walks the slots.  fp32 throughout, one rounding to the storage type.
template <typename T>
__global__ __launch_bounds__(64) void fwd_attend_plain_kernel(const void *Q_, const void *Kc_, const void *Vc_,
                                                              const int32_t *slot_pos, const int32_t *insert_slot,
                                                              const int32_t *rebuilt_pos, void *O_, int H, int K, int d,
                                                              int nq, int r, int Rdim, int n, float scale_log2) {
  extern __shared__ __align__(16) unsigned char smem[];
  float *s_w = reinterpret_cast<float *>(smem);   // [K] logit, then probability; < 0 marks nothing (see s_vis)
  int32_t *s_vis = reinterpret_cast<int32_t *>(s_w + K);   // [K] 1 = visible to this query
  const int bh = blockIdx.x / nq, j = blockIdx.x - bh * nq;
  const int b = bh / H, h = bh - b * H;
  const int lane = threadIdx.x;
  const int Hd = H * d;
  const int P = j < r ? rebuilt_pos[size_t(b) * Rdim + j] : n;   // this query's position
  const T *q = static_cast<const T *>(Q_) + (size_t(b) * nq + j) * Hd + h * d;
  const T *Kb = static_cast<const T *>(Kc_) + size_t(bh) * K * d;
  const T *Vb = static_cast<const T *>(Vc_) + size_t(bh) * K * d;
  const int32_t *sp = slot_pos + size_t(bh) * K;
  const int s_ins = insert_slot[bh];
  float mx = -INFINITY;
  for (int k = lane; k < K; k += 64) {
    const int pos = k == s_ins ? n : sp[k];
    const bool vis = pos >= 0 && pos <= P;
    float w = 0.f;
    if (vis) {
      for (int c = 0; c < d; ++c) w = fmaf(to_float(q[c]), to_float(Kb[size_t(k) * d + c]), w);
      mx = fmaxf(mx, w);
    }
    s_w[k] = w;
    s_vis[k] = vis ? 1 : 0;
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
  float l = 0.f;
  for (int k = lane; k < K; k += 64) {
    const float p = s_vis[k] ? exp2f((s_w[k] - mx) * scale_log2) : 0.f;
    s_w[k] = p;
    l += p;
  }
  l = wave_sum(l);
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");   // one wave: its LDS stores before its LDS loads below
  __builtin_amdgcn_wave_barrier();
  T *o = static_cast<T *>(O_) + (size_t(b) * nq + j) * Hd + h * d;
  for (int c = lane; c < d; c += 64) {
    float acc = 0.f;
    for (int k = 0; k < K; ++k)
      if (s_vis[k]) acc = fmaf(s_w[k], to_float(Vb[size_t(k) * d + c]), acc);
    store_elem(o + c, acc / l);
  }
}

}  // namespace

// Largest cache the forward attention takes: the slot positions of a row sit in LDS next to the tiles.
int fwd_attend_max_slots() { return 8192; }

// Whether the matrix-core kernel takes this configuration's forward attention (otherwise the plain kernel does).
bool fwd_attend_mfma(const adore_config &c) {
  return c.dtype == ADORE_BF16 && c.rebuild_budget + 1 <= 64 && (c.head_dim == 64 || c.head_dim == 128);
}

hipError_t launch_fwd_attend(adore_ctx *ctx, int layer, int r) {
  const adore_config &c = ctx->cfg;
  const size_t layer_elems = size_t(c.batch) * c.heads * c.cache_slots * c.head_dim;
  if (!fwd_attend_mfma(c)) {
    ScopedTimer t(ctx, ADORE_KERNEL_FWD_ATTEND, ctx->stream);
    const size_t es = elem_size(c);
    const dim3 grid(unsigned(c.batch * c.heads * (r + 1))), block(64);
    const int lds = c.cache_slots * 8;
    const float scale_log2 = 1.4426950408889634f / sqrtf(float(c.head_dim));
    const void *Kl = ctx->cache_k + layer * layer_elems * es, *Vl = ctx->cache_v + layer * layer_elems * es;
    if (c.dtype == ADORE_BF16) {
      ADORE_LAUNCH(t, (fwd_attend_plain_kernel<bf16_t>), grid, block, lds, ctx->stream, ctx->fwd_q, Kl, Vl,
                   ctx->slot_pos[ctx->cur], ctx->insert_slot[ctx->cur], ctx->rebuilt_pos[ctx->cur], ctx->fwd_o, c.heads,
                   c.cache_slots, c.head_dim, r + 1, r, max(c.rebuild_budget, 1), ctx->n, scale_log2);
    } else {
      ADORE_LAUNCH(t, (fwd_attend_plain_kernel<float>), grid, block, lds, ctx->stream, ctx->fwd_q, Kl, Vl,
                   ctx->slot_pos[ctx->cur], ctx->insert_slot[ctx->cur], ctx->rebuilt_pos[ctx->cur], ctx->fwd_o, c.heads,
                   c.cache_slots, c.head_dim, r + 1, r, max(c.rebuild_budget, 1), ctx->n, scale_log2);
    }
    return hipGetLastError();
  }
  FwdAttendArgs a;
  a.Q = static_cast<const bf16_t *>(ctx->fwd_q);
  a.Kc = reinterpret_cast<const bf16_t *>(ctx->cache_k) + layer * layer_elems;
  a.Vc = reinterpret_cast<const bf16_t *>(ctx->cache_v) + layer * layer_elems;
  a.slot_pos = ctx->slot_pos[ctx->cur];
  a.insert_slot = ctx->insert_slot[ctx->cur];
  a.rebuilt_pos = ctx->rebuilt_pos[ctx->cur];
  a.O = static_cast<bf16_t *>(ctx->fwd_o);
  a.H = c.heads; a.K = c.cache_slots; a.nq = r + 1; a.r = r; a.Rdim = max(c.rebuild_budget, 1); a.n = ctx->n;
  a.chunk = ((c.cache_slots + kFwdWaves - 1) / kFwdWaves + 31) / 32 * 32;
  a.Kp = a.chunk * kFwdWaves;
  a.scale_log2 = 1.4426950408889634f / sqrtf(float(c.head_dim));
  const int rows = c.batch * c.heads;
  return c.head_dim == 128 ? launch_dh<128>(ctx, a, rows) : launch_dh<64>(ctx, a, rows);
}

}  // namespace adore
