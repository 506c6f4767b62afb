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
// 16-byte vectors with no transposes.  128x128 output tile per workgroup, four
// waves of 64x64, BK = 64, LDS double-buffered and XOR-swizzled.
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

__device__ inline int swz(int row, int chunk) { return row * CH + (chunk ^ ((row >> 1) & 7)); }

template <int NS>   // register stages: tiles of k-steps ks+1 .. ks+NS are in flight while ks is multiplied
__global__ __launch_bounds__(256) void rebuild_mfma_kernel(const GemmArgs a) {
  __shared__ u32x4 sA[2][BM * CH];
  __shared__ u32x4 sB[2][BN * CH];

  // Workgroups are dealt round-robin to the 8 XCDs; give each XCD a contiguous run of
  // tiles in which the M-tiles of one W panel are neighbours, so a panel is fetched
  // into one L2 only.
  const int total = a.tiles_m * a.tiles_n;
  const int per_xcd = (total + 7) / 8;
  const int lin = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (lin >= total) return;
  const int tn = lin / a.tiles_m, tm = lin - tn * a.tiles_m;
  const int m0 = tm * BM, n0 = tn * BN;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;

  // ---- global -> register staging: 4 chunks of A and 4 of B per thread and k-step ----
  const int lchunk = tid & 7, lrow = tid >> 3;   // rows lrow + 32*i
  const u32x4 *gA[4], *gB[4];
  const bf16_t *X = static_cast<const bf16_t *>(a.X);
  const bf16_t *W = static_cast<const bf16_t *>(a.W);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int mi = m0 + lrow + 32 * i;
    size_t src_row = 0;   // rows past M read a valid row and are dropped in the epilogue
    if (mi < a.M) {
      const int b = mi / a.r, rho = mi - b * a.r;
      src_row = size_t(b) * a.N_max + a.rebuilt_pos[size_t(b) * a.Rdim + rho];
    }
    gA[i] = reinterpret_cast<const u32x4 *>(X + src_row * a.D) + lchunk;
    gB[i] = reinterpret_cast<const u32x4 *>(W + size_t(n0 + lrow + 32 * i) * a.D) + lchunk;
  }
  const int nk = a.D / BK;
  u32x4 ra[NS][4], rb[NS][4];
#define ADORE_GLOAD(SET, KS)                    \
  _Pragma("unroll") for (int i = 0; i < 4; ++i) { \
    ra[SET][i] = gA[i][(KS) * CH];              \
    rb[SET][i] = gB[i][(KS) * CH];              \
  }
#define ADORE_LSTORE(SET, ST)                                 \
  _Pragma("unroll") for (int i = 0; i < 4; ++i) {             \
    sA[ST][swz(lrow + 32 * i, lchunk)] = ra[SET][i];          \
    sB[ST][swz(lrow + 32 * i, lchunk)] = rb[SET][i];          \
  }
#pragma unroll
  for (int s = 0; s < NS; ++s) {
    if (s < nk) { ADORE_GLOAD(s, s) }
  }
  ADORE_LSTORE(0, 0)
  __syncthreads();

  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  for (int ks0 = 0; ks0 < nk; ks0 += NS) {
#pragma unroll
    for (int u = 0; u < NS; ++u) {
      const int ks = ks0 + u;   // nk is a multiple of NS (checked at launch)
      {
        const int st = ks & 1;
        // register set u went to LDS one step ago: refill it with the tile NS steps ahead
        if (ks + NS < nk) { ADORE_GLOAD(u, ks + NS) }
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
          const int ch = kk * 2 + (lane >> 5);
          bf16x8 fa[2], fb[2];
#pragma unroll
          for (int i = 0; i < 2; ++i) {
            const u32x4 va = sA[st][swz(wm * 64 + i * 32 + (lane & 31), ch)];
            const u32x4 vb = sB[st][swz(wn * 64 + i * 32 + (lane & 31), ch)];
            fa[i] = *reinterpret_cast<const bf16x8 *>(&va);
            fb[i] = *reinterpret_cast<const bf16x8 *>(&vb);
          }
#pragma unroll
          for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
              acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
        if (ks + 1 < nk) { ADORE_LSTORE((u + 1) % NS, st ^ 1) }
        __syncthreads();
      }
    }
  }

#undef ADORE_GLOAD
#undef ADORE_LSTORE
  // ---- epilogue: round once to bf16 and scatter into the assigned slots ----
  // accumulator element v of lane L: row 8*(v/4) + 4*(L/32) + v%4, column L%32 of its 32x32 block
  const int Hd = a.H * a.d;
  bf16_t *Kc = static_cast<bf16_t *>(a.Kc);
  bf16_t *Vc = static_cast<bf16_t *>(a.Vc);
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int nf = n0 + wn * 64 + j * 32 + (lane & 31);
    const int half = nf / Hd, rem = nf - half * Hd;
    const int h = rem / a.d, cc = rem - h * a.d;
    bf16_t *dst_base = half ? Vc : Kc;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int mi = m0 + wm * 64 + i * 32 + 8 * (v / 4) + 4 * (lane >> 5) + (v % 4);
        if (mi < a.M) {
          const int b = mi / a.r, rho = mi - b * a.r;
          const int slot = a.free_list[(size_t(b) * a.H + h) * a.R1 + rho];
          dst_base[((size_t(b) * a.H + h) * a.K + slot) * a.d + cc].bits = f32_to_bf16_rne(acc[i][j][v]);
        }
      }
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

hipError_t launch_rebuild_gemm(adore_ctx *ctx, int layer, const void *hidden_layer, int r) {
  const adore_config &c = ctx->cfg;
  if (r <= 0) return hipSuccess;
  const size_t es = elem_size(c);
  const size_t layer_bytes = size_t(c.batch) * c.heads * c.cache_slots * c.head_dim * es;
  GemmArgs a;
  a.X = hidden_layer;
  a.W = static_cast<const char *>(ctx->w.w_kv) + size_t(layer) * 2 * c.heads * c.head_dim * c.hidden * es;
  a.Kc = ctx->cache_k + layer * layer_bytes;
  a.Vc = ctx->cache_v + layer * layer_bytes;
  a.rebuilt_pos = ctx->rebuilt_pos;
  a.free_list = ctx->free_list;
  a.B = c.batch; a.H = c.heads; a.d = c.head_dim; a.D = c.hidden; a.K = c.cache_slots;
  a.N_max = c.max_positions; a.r = r; a.R1 = c.rebuild_budget + 1; a.Rdim = max(c.rebuild_budget, 1);
  a.M = c.batch * r; a.N = 2 * c.heads * c.head_dim;
  a.tiles_m = (a.M + BM - 1) / BM; a.tiles_n = a.N / BN;
  ScopedTimer t(ctx, ADORE_KERNEL_REBUILD_GEMM);
  const bool mfma_ok = c.dtype == ADORE_BF16 && c.hidden % BK == 0 && a.N % BN == 0 && c.head_dim % 32 == 0;
  if (mfma_ok) {
    const int total = a.tiles_m * a.tiles_n;
    const int grid = (total + 7) / 8 * 8;
    const int nk = c.hidden / BK;   // the k-loop is unrolled by the number of register stages
    if (nk % 4 == 0) hipLaunchKernelGGL((rebuild_mfma_kernel<4>), dim3(grid), dim3(256), 0, ctx->stream, a);
    else if (nk % 2 == 0) hipLaunchKernelGGL((rebuild_mfma_kernel<2>), dim3(grid), dim3(256), 0, ctx->stream, a);
    else hipLaunchKernelGGL((rebuild_mfma_kernel<1>), dim3(grid), dim3(256), 0, ctx->stream, a);
  } else {
    const size_t waves = size_t(a.M) * a.N;
    const unsigned blocks = unsigned((waves + 3) / 4);
    if (c.dtype == ADORE_BF16) {
      hipLaunchKernelGGL((rebuild_dot_kernel<bf16_t>), dim3(blocks), dim3(256), 0, ctx->stream, a);
    } else {
      hipLaunchKernelGGL((rebuild_dot_kernel<float>), dim3(blocks), dim3(256), 0, ctx->stream, a);
    }
  }
  return hipGetLastError();
}

}  // namespace adore
