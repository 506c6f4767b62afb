// Stage 4: rebuild the K/V states of the chosen released tokens (paper Sec. 2.3)
// by re-projecting their hidden states with W_k / W_v and writing each head's
// slice straight into the slot the schedule assigned to it.
//
//   C[M = B*r, N = 2*H*d] = X_gathered[M, D] * W_kv[N, D]^T     (fp32 accumulate, one rounding)
//
// Row mi of the product is token rho = mi % r of sequence b = mi / r; its source
// row is hidden[b][rebuilt_pos[b][rho]] (gather), its destination rows are
// cache_{k,v}[b][h][free_list[b][h][rho]] (scatter).  No [M,N] tensor is ever
// materialised and nothing is compacted.
//
// bf16 path: a real dense contraction, so it runs on the matrix cores
// (v_mfma_f32_32x32x16_bf16).  Both operands are contiguous along the reduction
// dimension, which is exactly the per-lane operand layout of that instruction
// (8 consecutive k for one row), so tiles go global -> LDS -> registers as
// 16-byte vectors with no transposes.  128x128 output tile per workgroup (one
// per compute unit at the 7B shape: M = 512, N = 8192), BK = 64, LDS
// triple-buffered and XOR-swizzled (conflict-free for 16-byte reads and writes).
// The output tile is rounded to bf16 into LDS and leaves as 16-byte vectors: a
// row of the tile is a contiguous head slice of one cache row.
// fp32 path (and shapes the tile kernel does not take): one wave per output.
#include "device_utils.h"

namespace adore {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // plain vector: stays in registers

struct GemmArgs {
  const void *X;               // [B][N_max][D] hidden states entering this layer
  const void *W;               // [N][D]
  void *Kc, *Vc;               // [B][H][K][d] of this layer
  const int32_t *rebuilt_pos;  // [B][Rdim]
  const int32_t *free_list;    // [B][H][R1]
  int B, H, d, D, K, N_max, r, R1, Rdim, M, N;
  int tiles_m, tiles_n;
};

constexpr int BM = 128, BN = 128, BK = 64;
constexpr int CH = BK / 8;   // 16-byte chunks per tile row
constexpr int LS = 3;        // LDS stages

__device__ inline int swz(int row, int chunk) { return row * CH + (chunk ^ ((row >> 1) & 7)); }

// Workgroup = 8 waves on a 128x128 output tile.  Waves 0-3 and 4-7 form two k-groups: each group
// holds the whole tile as four 64x64 wave tiles and multiplies one half of every 64-wide k-step, so
// the LDS read traffic is that of four waves while every SIMD has two waves to switch between.  The
// two halves are added through LDS at the end.
//   global -> registers: NS k-steps ahead (NS register sets, refilled right after they are spilled to LDS)
//   registers -> LDS:    three stages, so the tile of step ks+2 is written while ks is read and ks+1 is
//                        already complete; one barrier per k-step, and the first fragments of the next
//                        step are fetched before it
//   LDS -> fragments:    one 16-wide k-slice ahead of the MFMAs that use them
// sched_barrier keeps the compiler from sinking the fragment loads below the MFMAs they overlap with.
template <int NS>
__global__ __launch_bounds__(512) void rebuild_mfma_kernel(const GemmArgs a) {
  // one LDS block: LS stages of (A tile, B tile); after the k-loop the first 64 KB carry the upper
  // k-group's accumulators and the last 32 KB the bf16 output tile
  __shared__ u32x4 smem[LS * (BM + BN) * CH];
  __shared__ long long s_dst[BM * (BN / 64)];   // element offset of each output row slice in the cache, -1 = none
  u32x4 (*sA)[BM * CH] = reinterpret_cast<u32x4 (*)[BM * CH]>(smem);
  u32x4 (*sB)[BN * CH] = reinterpret_cast<u32x4 (*)[BN * CH]>(smem + LS * BM * CH);

  const int total = a.tiles_m * a.tiles_n;
  const int per_xcd = (total + 7) / 8;
  const int lin = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (lin >= total) return;
  const int tn = lin / a.tiles_m, tm = lin - tn * a.tiles_m;
  const int m0 = tm * BM, n0 = tn * BN;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int kgrp = wave >> 2, wm = (wave >> 1) & 1, wn = wave & 1;

  // where every row of the output tile goes: looked up now, used after the k-loop
  const int Hd = a.H * a.d;
  const int nh = BN / a.d > 0 ? BN / a.d : 1;     // heads covered by the tile's 128 columns (d = 64: 2, d >= 128: 1)
  if (tid < BM * nh) {
    const int row = tid / nh, hh = tid - row * nh;
    const int mi = m0 + row;
    long long off = -1;
    if (mi < a.M) {
      const int b = mi / a.r, rho = mi - b * a.r;
      const int nf = n0 + hh * a.d;
      const int rem = nf % Hd;
      const int h = rem / a.d;
      const int slot = a.free_list[(size_t(b) * a.H + h) * a.R1 + rho];
      off = ((long long)(size_t(b) * a.H + h) * a.K + slot) * a.d + (rem - h * a.d);
    }
    s_dst[tid] = off;
  }
  const int lchunk = tid & 7, lrow = tid >> 3;   // rows lrow + 64*i
  const u32x4 *gA[2], *gB[2];
  const bf16_t *X = static_cast<const bf16_t *>(a.X);
  const bf16_t *W = static_cast<const bf16_t *>(a.W);
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int mi = m0 + lrow + 64 * i;
    size_t src_row = 0;
    if (mi < a.M) {
      const int b = mi / a.r, rho = mi - b * a.r;
      src_row = size_t(b) * a.N_max + a.rebuilt_pos[size_t(b) * a.Rdim + rho];
    }
    gA[i] = reinterpret_cast<const u32x4 *>(X + src_row * a.D) + lchunk;
    gB[i] = reinterpret_cast<const u32x4 *>(W + size_t(n0 + lrow + 64 * i) * a.D) + lchunk;
  }
  const int nk = a.D / BK;
  u32x4 ra[NS][2], rb[NS][2];
#define GLOAD(SET, KS)                                              \
  _Pragma("unroll") for (int i = 0; i < 2; ++i) {                   \
    ra[SET][i] = gA[i][(KS) * CH];                                  \
    rb[SET][i] = gB[i][(KS) * CH];                                  \
  }
#define LSTORE(SET, ST)                                             \
  _Pragma("unroll") for (int i = 0; i < 2; ++i) {                   \
    sA[ST][swz(lrow + 64 * i, lchunk)] = ra[SET][i];                \
    sB[ST][swz(lrow + 64 * i, lchunk)] = rb[SET][i];                \
  }
#define FRAGS(FA, FB, ST, KK)                                                         \
  {                                                                                   \
    const int ch_ = (KK) * 2 + (lane >> 5);                                           \
    _Pragma("unroll") for (int i = 0; i < 2; ++i) {                                   \
      const u32x4 va_ = sA[ST][swz(wm * 64 + i * 32 + (lane & 31), ch_)];             \
      const u32x4 vb_ = sB[ST][swz(wn * 64 + i * 32 + (lane & 31), ch_)];             \
      FA[i] = *reinterpret_cast<const bf16x8 *>(&va_);                                \
      FB[i] = *reinterpret_cast<const bf16x8 *>(&vb_);                                \
    }                                                                                 \
  }
#define MFMA4(FA, FB)                                                                 \
  _Pragma("unroll") for (int i = 0; i < 2; ++i)                                       \
    _Pragma("unroll") for (int j = 0; j < 2; ++j)                                     \
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(FA[i], FB[j], acc[i][j], 0, 0, 0);

  // prologue: tiles 0 and 1 to LDS, tiles 2 .. NS+1 into the register sets (set of tile t = t % NS)
  GLOAD(0, 0)
  LSTORE(0, 0)
  if (nk > 1) {
    GLOAD(1 % NS, 1)
    LSTORE(1 % NS, 1)
  }
#pragma unroll
  for (int s = 0; s < NS; ++s) {
    if (s + 2 < nk) { GLOAD((s + 2) % NS, s + 2) }
  }
  __syncthreads();

  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  const int kk0 = 2 * kgrp, kk1 = 2 * kgrp + 1;
  bf16x8 fa0[2], fb0[2], fa1[2], fb1[2];
  FRAGS(fa0, fb0, 0, kk0)
  int st = 0;   // LDS stage of tile ks
  // One k-step.  IF(c) guards the parts that run out near the end; it is empty in the steady loop so
  // that the loop body is a single basic block (the wait counters are then tracked exactly).
#define KSTEP(U, KS, IF)                                                         \
  {                                                                              \
    const int st1 = st == LS - 1 ? 0 : st + 1;                                   \
    const int st2 = st1 == LS - 1 ? 0 : st1 + 1;                                 \
    FRAGS(fa1, fb1, st, kk1)                                                     \
    __builtin_amdgcn_sched_barrier(0);                                           \
    MFMA4(fa0, fb0)                                                              \
    __builtin_amdgcn_sched_barrier(0);                                           \
    IF((KS) + 2 < nk) { LSTORE(((U) + 2) % NS, st2) }                            \
    IF((KS) + 2 + NS < nk) { GLOAD(((U) + 2) % NS, (KS) + 2 + NS) }              \
    IF((KS) + 1 < nk) { FRAGS(fa0, fb0, st1, kk0) }                              \
    __builtin_amdgcn_sched_barrier(0);                                           \
    MFMA4(fa1, fb1)                                                              \
    __builtin_amdgcn_sched_barrier(0);                                           \
    __syncthreads();                                                             \
    st = st1;                                                                    \
  }
#define ALWAYS(c)
#define GUARDED(c) if (c)
  const int nk_main = nk >= NS + 2 ? (nk - NS - 2) / NS * NS : 0;   // k-steps that need no guard
  int ks0 = 0;
  for (; ks0 < nk_main; ks0 += NS) {
#pragma unroll
    for (int u = 0; u < NS; ++u) KSTEP(u, ks0 + u, ALWAYS)
  }
  for (; ks0 < nk; ks0 += NS) {
#pragma unroll
    for (int u = 0; u < NS; ++u) {
      if (ks0 + u < nk) KSTEP(u, ks0 + u, GUARDED)   // uniform over the workgroup: the barrier inside is safe
    }
  }
#undef KSTEP
#undef ALWAYS
#undef GUARDED
#undef GLOAD
#undef LSTORE
#undef FRAGS
#undef MFMA4

  // ---- add the two k-groups: the upper four waves hand their accumulators over through LDS ----
  float *red = reinterpret_cast<float *>(smem) + (wave & 3) * 64 * 64 + lane;   // 4 x 16 KB
  if (kgrp == 1) {
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) red[((i * 2 + j) * 16 + v) * 64] = acc[i][j][v];
  }
  __syncthreads();
  // ---- round once to bf16 into a row-major LDS tile ----
  // accumulator element v of lane L: row 8*(v/4) + 4*(L/32) + v%4, column L%32 of its 32x32 block
  uint16_t *sOut = reinterpret_cast<uint16_t *>(smem) + 64 * 1024 / 2;            // [BM][BN] bf16 = 32 KB
  if (kgrp == 0) {
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const float s = acc[i][j][v] + red[((i * 2 + j) * 16 + v) * 64];
          const int row = wm * 64 + i * 32 + 8 * (v / 4) + 4 * (lane >> 5) + (v % 4);
          const int col = wn * 64 + j * 32 + (lane & 31);
          sOut[row * BN + col] = f32_to_bf16_rne(s);
        }
  }
  __syncthreads();
  // ---- scatter: every output row slice is contiguous in the cache; 16 bytes per lane ----
  bf16_t *dst_half = static_cast<bf16_t *>(n0 >= Hd ? a.Vc : a.Kc);
#pragma unroll
  for (int i = 0; i < (BM * BN / 8) / 512; ++i) {
    const int idx = i * 512 + tid;
    const int row = idx >> 4, vec = idx & 15;            // 16 vectors of 8 columns per row
    const long long off = s_dst[row * nh + (vec * 8) / a.d];
    if (off >= 0) {
      const u32x4 val = *reinterpret_cast<const u32x4 *>(sOut + row * BN + vec * 8);
      *reinterpret_cast<u32x4 *>(dst_half + off + (vec * 8) % a.d) = val;
    }
  }
}

// One wave per output element: dot of a gathered hidden row with one W row.
template <typename T>
__global__ __launch_bounds__(256) void rebuild_dot_kernel(const GemmArgs a) {
  constexpr int EPL = Vec16<T>::EPL;
  const size_t wid = (size_t(blockIdx.x) * blockDim.x + threadIdx.x) >> 6;
  const int lane = threadIdx.x & 63;
  if (wid >= size_t(a.M) * a.N) return;
  const int mi = int(wid / a.N), nf = int(wid - size_t(mi) * a.N);
  const int b = mi / a.r, rho = mi - b * a.r;
  const int pos = a.rebuilt_pos[size_t(b) * a.Rdim + rho];
  const T *x = static_cast<const T *>(a.X) + (size_t(b) * a.N_max + pos) * a.D;
  const T *wrow = static_cast<const T *>(a.W) + size_t(nf) * a.D;
  float s = 0.f;
  for (int c = lane * EPL; c < a.D; c += 64 * EPL) {
    float xf[EPL], wf[EPL];
    Vec16<T>::load(x + c, xf);
    Vec16<T>::load(wrow + c, wf);
#pragma unroll
    for (int e = 0; e < EPL; ++e) s = fmaf(xf[e], wf[e], s);
  }
  s = wave_sum(s);
  if (lane == 0) {
    const int Hd = a.H * a.d;
    const int half = nf / Hd, rem = nf - half * Hd;
    const int h = rem / a.d, cc = rem - h * a.d;
    const int slot = a.free_list[(size_t(b) * a.H + h) * a.R1 + rho];
    T *dst = static_cast<T *>(half ? a.Vc : a.Kc) + ((size_t(b) * a.H + h) * a.K + slot) * a.d + cc;
    store_elem(dst, s);
  }
}

}  // namespace

hipError_t launch_rebuild_gemm(adore_ctx *ctx, int layer, const void *hidden_layer, int lists, int r) {
  const adore_config &c = ctx->cfg;
  if (r <= 0) return hipSuccess;
  const size_t es = elem_size(c);
  const size_t layer_bytes = size_t(c.batch) * c.heads * c.cache_slots * c.head_dim * es;
  GemmArgs a;
  a.X = hidden_layer;
  a.W = static_cast<const char *>(ctx->w.w_kv) + size_t(layer) * 2 * c.heads * c.head_dim * c.hidden * es;
  a.Kc = ctx->cache_k + layer * layer_bytes;
  a.Vc = ctx->cache_v + layer * layer_bytes;
  a.rebuilt_pos = ctx->rebuilt_pos[lists];
  a.free_list = ctx->free_list[lists];
  a.B = c.batch; a.H = c.heads; a.d = c.head_dim; a.D = c.hidden; a.K = c.cache_slots;
  a.N_max = c.max_positions; a.r = r; a.R1 = c.rebuild_budget + 1; a.Rdim = max(c.rebuild_budget, 1);
  a.M = c.batch * r; a.N = 2 * c.heads * c.head_dim;
  a.tiles_m = (a.M + BM - 1) / BM; a.tiles_n = a.N / BN;
  ScopedTimer t(ctx, ADORE_KERNEL_REBUILD_GEMM, ctx->stream);
  const bool mfma_ok = c.dtype == ADORE_BF16 && c.hidden % BK == 0 && (c.heads * c.head_dim) % BN == 0 &&
                       (BN % c.head_dim == 0 || c.head_dim % BN == 0);
  if (mfma_ok) {
    const int total = a.tiles_m * a.tiles_n;
    const int grid = (total + 7) / 8 * 8;
    const int nk = c.hidden / BK;   // the k-loop is unrolled by the number of register stages
    if (nk % 4 == 0) ADORE_LAUNCH(t, (rebuild_mfma_kernel<4>), dim3(grid), dim3(512), 0, ctx->stream, a);
    else if (nk % 2 == 0) ADORE_LAUNCH(t, (rebuild_mfma_kernel<2>), dim3(grid), dim3(512), 0, ctx->stream, a);
    else ADORE_LAUNCH(t, (rebuild_mfma_kernel<1>), dim3(grid), dim3(512), 0, ctx->stream, a);
  } else {
    const size_t waves = size_t(a.M) * a.N;
    const unsigned blocks = unsigned((waves + 3) / 4);
    if (c.dtype == ADORE_BF16) {
      ADORE_LAUNCH(t, (rebuild_dot_kernel<bf16_t>), dim3(blocks), dim3(256), 0, ctx->stream, a);
    } else {
      ADORE_LAUNCH(t, (rebuild_dot_kernel<float>), dim3(blocks), dim3(256), 0, ctx->stream, a);
    }
  }
  return hipGetLastError();
}

}  // namespace adore
