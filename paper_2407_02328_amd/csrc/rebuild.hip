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
// 16-byte vectors with no transposes.  One kernel template covers a family of
// output tiles; the launcher takes the largest tile that still gives every compute
// unit a workgroup (M = 512 at the 7B shape: 128x128, one tile per unit;
// M >= 2048: 256x256; M <= 128: 128x32).  Larger tiles move fewer bytes per flop, from the
// L2 to the compute unit and through LDS, and that path is what the 128x128 tile runs into first.  LDS stages
// are XOR-swizzled (conflict-free for 16-byte reads and writes).  The output tile
// is rounded to bf16 into LDS and leaves as 16-byte vectors: a row of the tile is
// a run of contiguous head slices of cache rows.
// fp32 path (and shapes the tile kernel does not take): one wave per output.
#include "device_utils.h"

namespace adore {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // plain vector: stays in registers

// The same tile kernel serves the three projections of the path:
//   REBUILD  C = X[b][rebuilt_pos] . W_kv^T         -> head slices scattered into the freed cache slots
//   QKV      C = X_rows . [W_q ; W_kv]^T            -> query rows to a dense buffer, K/V slices scattered into the
//            slots of the rebuilt tokens and of the current token (rebuild forward, Sec. 2.3)
//   OPROJ    C = O_rows . W_o^T + X_rows (residual) -> dense rows, the next layer's input
// and one more product of the same shape family, the controller's input projection over a prompt chunk:
//   PLAIN    C = X_rows . W^T                        -> dense fp32 rows, no rounding
enum { MODE_REBUILD = 0, MODE_QKV = 1, MODE_OPROJ = 2, MODE_PLAIN = 3 };

struct GemmArgs {
  const void *X;               // A operand: [B][N_max][D] gathered by position, or dense rows [M][D]
  const void *W;               // [N][D]  (QKV: W_kv, the rows of columns >= H*d)
  const void *Wq;              // QKV: [H*d][D], the rows of columns < H*d
  void *Kc, *Vc;               // [B][H][K][d] of this layer
  void *Out;                   // QKV: query rows [M][H*d]; OPROJ: output rows [.][N]; PLAIN: fp32 rows [M][N]
  const void *Res;             // OPROJ: residual rows, gathered by position or dense like X
  const int32_t *rebuilt_pos;  // [B][Rdim]
  const int32_t *free_list;    // [B][H][R1]
  const int32_t *insert_slot;  // [B][H]    QKV: the slot of the current token
  int32_t *map_dst, *map_out;  // REBUILD: slot maps [B][H][K] that get the rebuilt tokens' positions, or null
  int B, H, d, D, K, N_max, r, R1, Rdim, M, N;   // D = length of the contraction
  int tiles_m, tiles_n;
  // Rows.  The tile kernel takes the rebuilt tokens: row mi = (b, j) = (mi / r, mi % r), rank j of sequence b.
  // The current token of every sequence (one row each) goes through cur_rows_kernel.  Dense row buffers hold
  // xrps rows per sequence: rank j at row b * xrps + j, the current token at row b * xrps + r.
  int xrps;
  int cur_pos;                 // position of the current token
  int a_gather, res_gather;    // 1: the row of a token is [b][its position]; 0: its row in a dense buffer
  int out_rps, out_cur;        // OPROJ: rank j is written to row b * out_rps + j, the current token to b * out_rps + out_cur
  int n_cur;                   // QKV / OPROJ: the first n_cur workgroups of the tile launch take the current tokens' rows
  int cur_ks;                  // ... with the contraction cut over cur_ks (1, 2, 4, 8) of a workgroup's waves
  const float2 *rope_cur;      // QKV: the workgroups of the current tokens' rows turn their query and key rows (same
                               // table; null: they do not)
  const float2 *rope;          // tile kernel: [N_max][d/2] (cos, sin), the key (and query) tiles turn their rows by
                               // position as they leave; null: no rotary embedding, or a pass of its own does it
};

// A rank that stays empty (position -1: fewer tokens were chosen than the launch has rows for) reads row 0 of its
// sequence; nothing of it is written.
__device__ inline size_t row_by_position(const GemmArgs &a, int b, int j) {
  return size_t(b) * a.N_max + max(a.rebuilt_pos[size_t(b) * a.Rdim + j], 0);
}

// The current token's row of every sequence (rebuild forward) as workgroups of the tile kernel's launch.  B rows
// against the same weights are a skinny product that only streams W; the tile launches of the forward leave a
// fifth or more of the compute units without a tile, and these workgroups take them (one workgroup per unit:
// the kernel's LDS sees to that), so the rows cost no launch and no time of their own.  A wave multiplies 16
// sequences x 32 output columns; the 8 waves of a workgroup are cur_ks wide along the contraction and 8 / cur_ks
// wide along the columns (partial sums added through LDS in a fixed order), so that the launcher can make as
// many workgroups as there are units without a tile: what one unit can stream is bounded by what it can keep
// in flight (about 36 GB/s next to the tiles' traffic).  With so few units at work the rows of W must arrive as whole cache lines (operands loaded
// straight into the 16x16x32 operand layout cost the L1 a tag look-up per lane, about 25 GB/s per unit): a wave
// reads its 32 rows x 64 k as four coalesced 16-byte loads per lane, six such chunks in flight, and turns them
// into operands through 4 KB of LDS of its own (XOR-swizzled; only the wave itself reads and writes it, so no
// barrier).  Epilogue as in the tile kernel, one rounding.
constexpr int kCurCols = 256;   // output columns per workgroup in this role when the contraction is not cut

template <int MODE>
__device__ inline void cur_rows_role(const GemmArgs &a, int e, u32x4 *smem) {
  typedef float f32x4 __attribute__((ext_vector_type(4)));
  constexpr int U = 6;                                  // chunks of 64 k in flight
  const int ks = a.cur_ks;
  const int wg_cols = kCurCols / ks;
  const int wgs_n = a.N / wg_cols;
  const int sb = e / wgs_n, jn = e - sb * wgs_n;
  const int t0 = sb * 16;
  if (t0 >= a.B) return;                                // workgroups that only pad the launch
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int c = lane & 15, g = lane >> 4;
  const int kpart = wave % ks;                          // this wave's part of the contraction
  const int j0 = jn * wg_cols + (wave / ks) * 32;
  const int Hd = a.H * a.d;
  const int bb = min(t0 + c, a.B - 1);                  // padded rows read a valid sequence; dropped at the store
  const size_t xrow = a.a_gather ? size_t(bb) * a.N_max + a.cur_pos : size_t(bb) * a.xrps + a.r;
  const u32x4 *pa = reinterpret_cast<const u32x4 *>(static_cast<const bf16_t *>(a.X) + xrow * a.D) + g;
  // W: lane (row8 = lane / 8, chunk = lane % 8) loads 16 bytes of row 8 i + row8 of the wave's 32 rows
  const int lrow = lane >> 3, lch = lane & 7;
  const u32x4 *pw[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int n = j0 + 8 * i + lrow;
    const bf16_t *wrow = MODE == MODE_QKV && n < Hd ? static_cast<const bf16_t *>(a.Wq) + size_t(n) * a.D
                         : MODE == MODE_QKV         ? static_cast<const bf16_t *>(a.W) + size_t(n - Hd) * a.D
                                                    : static_cast<const bf16_t *>(a.W) + size_t(n) * a.D;
    pw[i] = reinterpret_cast<const u32x4 *>(wrow) + lch;
  }
  u32x4 *tile = smem + wave * (32 * 8);                 // [32 rows][8 chunks of 16 bytes]
  auto swz = [](int row, int chunk) { return row * 8 + (chunk ^ ((row >> 1) & 7)); };
  f32x4 acc[2] = {f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}};
  const int nchunks = a.D / 64 / ks;                    // chunks of this wave: kpart * nchunks ...
  const int chunk0 = kpart * nchunks;
  u32x4 vw[U][4], va[U][2];
#define CUR_LOAD(SET, CH)                                                                \
  {                                                                                      \
    _Pragma("unroll") for (int i = 0; i < 4; ++i) vw[SET][i] = pw[i][(chunk0 + (CH)) * 8]; \
    va[SET][0] = pa[(chunk0 + (CH)) * 8];                                                \
    va[SET][1] = pa[(chunk0 + (CH)) * 8 + 4];                                            \
  }
#pragma unroll
  for (int u = 0; u < U; ++u) {
    if (u < nchunks) CUR_LOAD(u, u)
  }
  for (int ch0 = 0; ch0 < nchunks; ch0 += U) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int ch = ch0 + u;
      if (ch < nchunks) {
#pragma unroll
        for (int i = 0; i < 4; ++i) tile[swz(8 * i + lrow, lch)] = vw[u][i];
        u32x4 fb[2][2];   // [step of 32 k][tile of 16 columns]
#pragma unroll
        for (int st = 0; st < 2; ++st)
#pragma unroll
          for (int nc = 0; nc < 2; ++nc) fb[st][nc] = tile[swz(nc * 16 + c, st * 4 + g)];
        const u32x4 fa0 = va[u][0], fa1 = va[u][1];
        if (ch + U < nchunks) CUR_LOAD(u, ch + U)
#pragma unroll
        for (int nc = 0; nc < 2; ++nc) {
          acc[nc] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*reinterpret_cast<const bf16x8 *>(&fa0),
                                                            *reinterpret_cast<const bf16x8 *>(&fb[0][nc]), acc[nc], 0, 0, 0);
          acc[nc] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*reinterpret_cast<const bf16x8 *>(&fa1),
                                                            *reinterpret_cast<const bf16x8 *>(&fb[1][nc]), acc[nc], 0, 0, 0);
        }
      }
    }
  }
#undef CUR_LOAD
  const bool turning = MODE == MODE_QKV && a.rope_cur != nullptr;   // uniform over the launch
  if (ks > 1) {   // the parts of the contraction meet in the wave that holds part 0, in order
    float *red = reinterpret_cast<float *>(smem + 8 * (32 * 8));   // [8 waves][2][4][64], behind the waves' tiles
#pragma unroll
    for (int nc = 0; nc < 2; ++nc)
#pragma unroll
      for (int v = 0; v < 4; ++v) red[((wave * 2 + nc) * 4 + v) * 64 + lane] = acc[nc][v];
    __syncthreads();
    if (kpart != 0 && !turning) return;   // (when the rows are turned below, every wave stays for the barrier)
    for (int p = 1; p < (kpart == 0 ? ks : 1); ++p)
#pragma unroll
      for (int nc = 0; nc < 2; ++nc)
#pragma unroll
        for (int v = 0; v < 4; ++v) acc[nc][v] += red[(((wave + p) * 2 + nc) * 4 + v) * 64 + lane];
  }
  if (turning) {
    // Rotary embedding: the workgroup's columns are whole heads of one section (launcher).  The rounded results meet
    // in an LDS tile [16 sequences][wg_cols]; then a thread takes 8 planes at a time (the 8-element vectors of
    // elements j.. and j + d/2.. of a head), turns query and key rows to the current position, and stores 16 bytes.
    uint16_t *sT = reinterpret_cast<uint16_t *>(smem + 8 * (32 * 8) + 8 * 2 * 4 * 64 / 4);   // behind tiles and sums
    if (kpart == 0) {
#pragma unroll
      for (int v = 0; v < 4; ++v)
#pragma unroll
        for (int nc = 0; nc < 2; ++nc)
          sT[(4 * g + v) * wg_cols + (wave / ks) * 32 + nc * 16 + c] = f32_to_bf16_rne(acc[nc][v]);
    }
    __syncthreads();
    const int section = (jn * wg_cols) / Hd;             // 0: queries, 1: keys, 2: values
    const int half = a.d / 2;
    const bool turn = section <= 1;
    const int upr = turn ? wg_cols / 16 : wg_cols / 8;   // units per sequence: vector pairs, or single vectors
    for (int idx = tid; idx < 16 * upr; idx += 512) {
      const int seq = idx / upr, uu = idx - seq * upr;
      const int b = t0 + seq;
      if (b >= a.B) continue;
      int col, jp = 0;
      if (turn) {
        const int hv = half / 8, hh = uu / hv;
        jp = (uu - hh * hv) * 8;
        col = hh * a.d + jp;
      } else {
        col = uu * 8;
      }
      const int rem = jn * wg_cols + col - section * Hd;
      const int h = rem / a.d;
      bf16_t *dst;
      if (section == 0) {
        dst = static_cast<bf16_t *>(a.Out) + (size_t(b) * a.xrps + a.r) * Hd + rem;
      } else {
        const int slot = a.insert_slot[size_t(b) * a.H + h];
        dst = static_cast<bf16_t *>(section == 1 ? a.Kc : a.Vc) + ((size_t(b) * a.H + h) * a.K + slot) * a.d + (rem - h * a.d);
      }
      const u32x4 lo = *reinterpret_cast<const u32x4 *>(sT + seq * wg_cols + col);
      if (!turn) {
        *reinterpret_cast<u32x4 *>(dst) = lo;
        continue;
      }
      const u32x4 hi = *reinterpret_cast<const u32x4 *>(sT + seq * wg_cols + col + half);
      const float2 *cs = a.rope_cur + size_t(a.cur_pos) * half + jp;
      uint32_t rl[8], rh[8];
#pragma unroll
      for (int e2 = 0; e2 < 8; ++e2) {
        const float x = __uint_as_float(((lo[e2 / 2] >> (16 * (e2 & 1))) & 0xffffu) << 16);
        const float y = __uint_as_float(((hi[e2 / 2] >> (16 * (e2 & 1))) & 0xffffu) << 16);
        rl[e2] = f32_to_bf16_rne(rope_lo(x, y, cs[e2]));
        rh[e2] = f32_to_bf16_rne(rope_hi(x, y, cs[e2]));
      }
      *reinterpret_cast<u32x4 *>(dst) = u32x4{rl[0] | (rl[1] << 16), rl[2] | (rl[3] << 16), rl[4] | (rl[5] << 16), rl[6] | (rl[7] << 16)};
      *reinterpret_cast<u32x4 *>(dst + half) =
          u32x4{rh[0] | (rh[1] << 16), rh[2] | (rh[3] << 16), rh[4] | (rh[5] << 16), rh[6] | (rh[7] << 16)};
    }
    return;
  }
  // accumulator element v of lane (c, g): sequence 4*g + v of the block, column c of the tile
#pragma unroll
  for (int v = 0; v < 4; ++v) {
    const int b = t0 + 4 * g + v;
    if (b >= a.B) continue;
#pragma unroll
    for (int nc = 0; nc < 2; ++nc) {
      float val = acc[nc][v];
      const int n = j0 + nc * 16 + c;
      bf16_t *dst;
      if (MODE == MODE_OPROJ) {
        const size_t rrow = a.res_gather ? size_t(b) * a.N_max + a.cur_pos : size_t(b) * a.xrps + a.r;
        val += to_float(static_cast<const bf16_t *>(a.Res)[rrow * a.N + n]);
        dst = static_cast<bf16_t *>(a.Out) + (size_t(b) * a.out_rps + a.out_cur) * a.N + n;
      } else {
        const int section = n / Hd, rem = n - section * Hd;
        const int h = rem / a.d;
        if (section == 0) {
          dst = static_cast<bf16_t *>(a.Out) + (size_t(b) * a.xrps + a.r) * Hd + rem;
        } else {
          const int slot = a.insert_slot[size_t(b) * a.H + h];
          dst = static_cast<bf16_t *>(section == 1 ? a.Kc : a.Vc) + ((size_t(b) * a.H + h) * a.K + slot) * a.d + (rem - h * a.d);
        }
      }
      dst->bits = f32_to_bf16_rne(val);
    }
  }
}

// Workgroup = 8 waves on a BM x BN output tile, k-steps of BK.
//   KG = 1: the waves form a WM x WN grid, each holding (BM/WM) x (BN/WN) of the tile.
//   KG = 2: two such grids of four waves (k-groups); each multiplies one half of every k-step, so the
//           LDS read traffic is that of four waves while every SIMD still has two waves to switch
//           between.  The halves are added through LDS at the end.
//   global -> registers: NS k-steps ahead (NS register sets, refilled right after they are spilled to LDS)
//   registers -> LDS:    LS stages; the tile of step ks+LS-1 is written while ks is read, one barrier per
//                        k-step.  With LS >= 3 the tile of ks+1 is complete during ks, so the first
//                        fragments of the next step are fetched before the barrier.
//   LDS -> fragments:    one 16-wide k-slice ahead of the MFMAs that use them
// sched_barrier keeps the compiler from sinking the fragment loads below the MFMAs they overlap with.
template <int MODE, int BM, int BN, int BK, int KG, int WM, int WN, int LS, int NS>
__global__ __launch_bounds__(512) void rebuild_mfma_kernel(const GemmArgs a) {
  constexpr int CH = BK / 8;             // 16-byte chunks per tile row
  constexpr int RPP = 512 / CH;          // tile rows the workgroup loads per pass
  constexpr int TM = BM / (WM * 32), TN = BN / (WN * 32);   // 32x32 blocks per wave
  static_assert(KG * WM * WN == 8 && (KG == 1 || KG == 2), "eight waves");
  static_assert(TM * WM * 32 == BM && TN * WN * 32 == BN, "tile shape");
  constexpr int NA = BM / RPP, NB = (BN + RPP - 1) / RPP;   // 16-byte loads per thread and k-step
  static_assert(NA * RPP == BM && (NB * RPP == BN || BN < RPP), "tile rows");
  constexpr int KSUB = BK / 16 / KG;     // 16-wide k-slices per wave and k-step
  static_assert(KSUB == 2 || KSUB == 4, "fragment double buffering needs an even number of k-slices");
  constexpr int LEAD = LS - 1;
  constexpr int STAGE = (BM + BN) * CH;  // 16-byte units per LDS stage
  constexpr int LOOP_BYTES = LS * STAGE * 16;
  constexpr int RED_BYTES = KG == 2 ? 4 * TM * TN * 16 * 64 * 4 : 0;
  constexpr int OUT_BYTES = BM * BN * 2;
  constexpr int SMEM_BYTES = LOOP_BYTES > RED_BYTES ? (LOOP_BYTES > OUT_BYTES ? LOOP_BYTES : OUT_BYTES)
                                                    : (RED_BYTES > OUT_BYTES ? RED_BYTES : OUT_BYTES);
  constexpr int NH_MAX = BN / 64 > 0 ? BN / 64 : 1;
  // one LDS block: the stages during the k-loop, then the upper k-group's accumulators, then the bf16 output tile
  __shared__ u32x4 smem[SMEM_BYTES / 16];
  __shared__ long long s_dst[BM * NH_MAX];   // element offset of each output row slice in its destination, -1 = none
  __shared__ long long s_res[MODE == MODE_OPROJ ? BM : 1];   // element offset of each row's residual, -1 = none
  __shared__ int s_rpos[MODE == MODE_REBUILD || MODE == MODE_QKV ? BM : 1];   // position of each row's token
  // rows are 128 B (BK = 64) or 64 B (BK = 32): 16 consecutive rows at one chunk index hit 16 different bank groups
  auto swz = [](int row, int chunk) { return row * CH + (chunk ^ (CH == 8 ? (row >> 1) & 7 : (row >> 2) & 3)); };

  int bx = blockIdx.x;
  if constexpr (MODE == MODE_QKV || MODE == MODE_OPROJ) {
    if (bx < a.n_cur) {   // uniform over the workgroup; n_cur is a multiple of 8, so the tiles keep their XCDs
      cur_rows_role<MODE>(a, bx, smem);
      return;
    }
    bx -= a.n_cur;
  }
  const int total = a.tiles_m * a.tiles_n;
  const int per_xcd = (total + 7) / 8;
  const int lin = (bx & 7) * per_xcd + (bx >> 3);
  if (lin >= total) return;
  const int tn = lin / a.tiles_m, tm = lin - tn * a.tiles_m;
  const int m0 = tm * BM, n0 = tn * BN;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int kgrp = wave / (WM * WN), wm = (wave / WN) % WM, wn = wave % WN;

  const int Hd = a.H * a.d;
  const int lchunk = tid % CH, lrow = tid / CH;   // rows lrow + RPP*i
  const bool b_on = BN >= RPP || lrow < BN;       // narrow tiles: only some threads load W rows
  const u32x4 *gA[NA], *gB[NB];
  const bf16_t *X = static_cast<const bf16_t *>(a.X);
  const bf16_t *W = MODE == MODE_QKV ? (n0 < Hd ? static_cast<const bf16_t *>(a.Wq) + size_t(n0) * a.D
                                                  : static_cast<const bf16_t *>(a.W) + size_t(n0 - Hd) * a.D)
                                     : static_cast<const bf16_t *>(a.W) + size_t(n0) * a.D;
#pragma unroll
  for (int i = 0; i < NB; ++i) {
    const int nrow = b_on ? lrow + RPP * i : 0;
    gB[i] = reinterpret_cast<const u32x4 *>(W + size_t(nrow) * a.D) + lchunk;
  }
  const int nk = a.D / BK;
  u32x4 ra[NS][NA], rb[NS][NB];
#define SA(ST) (smem + (ST) * STAGE)
#define SB(ST) (smem + (ST) * STAGE + BM * CH)
#define GLOAD_A(SET, KS) { _Pragma("unroll") for (int i = 0; i < NA; ++i) ra[SET][i] = gA[i][(KS) * CH]; }
#define GLOAD_B(SET, KS) { _Pragma("unroll") for (int i = 0; i < NB; ++i) rb[SET][i] = gB[i][(KS) * CH]; }
#define GLOAD(SET, KS) { GLOAD_A(SET, KS) GLOAD_B(SET, KS) }
#define LSTORE(SET, ST)                                                                  \
  {                                                                                      \
    _Pragma("unroll") for (int i = 0; i < NA; ++i)                                       \
      SA(ST)[swz(lrow + RPP * i, lchunk)] = ra[SET][i];                                  \
    if (b_on) {                                                                          \
      _Pragma("unroll") for (int i = 0; i < NB; ++i)                                     \
        SB(ST)[swz(lrow + RPP * i, lchunk)] = rb[SET][i];                                \
    }                                                                                    \
  }
#define FRAGS(BUF, ST, KK)                                                               \
  {                                                                                      \
    const int ch_ = (KK) * 2 + (lane >> 5);                                              \
    _Pragma("unroll") for (int i = 0; i < TM; ++i) {                                     \
      const u32x4 va_ = SA(ST)[swz((wm * TM + i) * 32 + (lane & 31), ch_)];              \
      fa[BUF][i] = *reinterpret_cast<const bf16x8 *>(&va_);                              \
    }                                                                                    \
    _Pragma("unroll") for (int j = 0; j < TN; ++j) {                                     \
      const u32x4 vb_ = SB(ST)[swz((wn * TN + j) * 32 + (lane & 31), ch_)];              \
      fb[BUF][j] = *reinterpret_cast<const bf16x8 *>(&vb_);                              \
    }                                                                                    \
  }
#define MFMAS(BUF)                                                                       \
  _Pragma("unroll") for (int i = 0; i < TM; ++i)                                         \
    _Pragma("unroll") for (int j = 0; j < TN; ++j)                                       \
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[BUF][i], fb[BUF][j], acc[i][j], 0, 0, 0);

  // prologue: tiles 0 .. LEAD-1 to LDS, tiles LEAD .. LEAD+NS-1 into the register sets (set of tile t = t % NS).
  // Everything read from memory here is issued before anything is waited for: the W rows of the first NS tiles
  // (they depend on nothing), the positions of the gathered rows, the A rows, the destination slots.  (A read of
  // what the previous kernel wrote takes a microsecond or two; one after the other they cost a tenth of the launch.)
#pragma unroll
  for (int t = 0; t < NS; ++t) {
    if (t < nk) { GLOAD_B(t, t) }
  }
#pragma unroll
  for (int i = 0; i < NA; ++i) {
    const int mi = m0 + lrow + RPP * i;
    size_t src_row = 0;
    if (mi < a.M) {
      const int b = mi / a.r, j = mi - b * a.r;
      src_row = a.a_gather ? row_by_position(a, b, j) : size_t(b) * a.xrps + j;
    }
    gA[i] = reinterpret_cast<const u32x4 *>(X + src_row * a.D) + lchunk;
  }
#pragma unroll
  for (int t = 0; t < NS; ++t) {
    if (t < nk) { GLOAD_A(t, t) }
  }
  // where every row of the output tile goes: looked up now, used after the k-loop
  const int sw = MODE == MODE_OPROJ ? BN : a.d;   // width of a contiguous piece of an output row
  const int nh = BN / sw > 0 ? BN / sw : 1;       // pieces in one tile row
  const int section = MODE == MODE_OPROJ ? 0 : n0 / Hd;   // REBUILD: K, V; QKV: Q, K, V (a tile lies in one)
  for (int t = tid; MODE != MODE_PLAIN && t < BM * nh; t += 512) {
    const int row = t / nh, hh = t - row * nh;
    const int mi = m0 + row;
    long long off = -1;
    if (mi < a.M) {
      const int b = mi / a.r, j = mi - b * a.r;
      if (MODE == MODE_OPROJ) {
        off = (long long)(size_t(b) * a.out_rps + j) * a.N + n0;
      } else {
        const int rem = (n0 + hh * a.d) % Hd;
        const int h = rem / a.d;
        if (MODE == MODE_QKV && section == 0) {
          off = (long long)(size_t(b) * a.xrps + j) * Hd + rem;
        } else {
          const int slot = a.free_list[(size_t(b) * a.H + h) * a.R1 + j];
          off = ((long long)(size_t(b) * a.H + h) * a.K + slot) * a.d + (rem - h * a.d);
          // no slot: the head still holds this token's row (heads with maps of their own), or the rank is empty
          if (MODE == MODE_REBUILD && (slot < 0 || a.rebuilt_pos[size_t(b) * a.Rdim + j] < 0)) off = -1;
          if (MODE == MODE_REBUILD && a.map_dst && section == 0) {   // the K half's tiles visit every (token, head)
            const int pos = a.rebuilt_pos[size_t(b) * a.Rdim + j];
            a.map_dst[(size_t(b) * a.H + h) * a.K + slot] = pos;
            if (a.map_out) a.map_out[(size_t(b) * a.H + h) * a.K + slot] = pos;
          }
        }
      }
    }
    s_dst[t] = off;
  }
  if ((MODE == MODE_REBUILD || MODE == MODE_QKV) && a.rope) {
    for (int row = tid; row < BM; row += 512) {
      const int mi = min(m0 + row, a.M - 1);
      s_rpos[row] = max(a.rebuilt_pos[size_t(mi / a.r) * a.Rdim + (mi % a.r)], 0);
    }
  }
  if (MODE == MODE_OPROJ) {
    for (int row = tid; row < BM; row += 512) {
      const int mi = m0 + row;
      long long ro = -1;
      if (mi < a.M) {
        const int b = mi / a.r, j = mi - b * a.r;
        ro = (long long)(a.res_gather ? row_by_position(a, b, j) : size_t(b) * a.xrps + j) * a.N + n0;
      }
      s_res[row] = ro;
    }
  }
#pragma unroll
  for (int t = 0; t < LEAD; ++t) {
    if (t < nk) { LSTORE(t % NS, t) }
    if (t + NS < nk) { GLOAD(t % NS, t + NS) }   // the set just stored takes the tile NS further on
  }
  __syncthreads();

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  const int kbase = KSUB * kgrp;   // first k-slice of this wave's k-group
  bf16x8 fa[2][TM], fb[2][TN];     // double-buffered fragments
  FRAGS(0, 0, kbase)
  int st = 0;                      // LDS stage of tile ks
  // One k-step.  IF(c) guards the parts that run out near the end; it is empty in the steady loop so
  // that the loop body is a single basic block (the wait counters are then tracked exactly).
#define KSTEP(U, KS, IF)                                                                 \
  {                                                                                      \
    const int st1 = st == LS - 1 ? 0 : st + 1;                                           \
    const int stw = st + LEAD >= LS ? st + LEAD - LS : st + LEAD;                        \
    _Pragma("unroll") for (int kk = 0; kk < KSUB; ++kk) {                                \
      if (kk + 1 < KSUB) {                                                               \
        FRAGS((kk + 1) & 1, st, kbase + kk + 1)                                          \
      } else if (LS > 2) {                                                               \
        IF((KS) + 1 < nk) { FRAGS(0, st1, kbase) }                                       \
      }                                                                                  \
      __builtin_amdgcn_sched_barrier(0);                                                 \
      MFMAS(kk & 1)                                                                      \
      __builtin_amdgcn_sched_barrier(0);                                                 \
      if (kk == 0) {                                                                     \
        IF((KS) + LEAD < nk) { LSTORE(((U) + LEAD) % NS, stw) }                          \
        IF((KS) + LEAD + NS < nk) { GLOAD(((U) + LEAD) % NS, (KS) + LEAD + NS) }         \
      }                                                                                  \
    }                                                                                    \
    __syncthreads();                                                                     \
    if (LS == 2) { IF((KS) + 1 < nk) { FRAGS(0, st1, kbase) } }                          \
    st = st1;                                                                            \
  }
#define ALWAYS(c)
#define GUARDED(c) if (c)
  const int nk_main = nk >= NS + LEAD ? (nk - NS - LEAD) / NS * NS : 0;   // k-steps that need no guard
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
#undef GLOAD_A
#undef GLOAD_B
#undef LSTORE
#undef FRAGS
#undef MFMAS
#undef SA
#undef SB

  // ---- add the two k-groups: the upper four waves hand their accumulators over through LDS ----
  if (KG == 2) {
    float *red = reinterpret_cast<float *>(smem) + (wave % (WM * WN)) * (TM * TN * 16 * 64) + lane;
    if (kgrp == 1) {
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int v = 0; v < 16; ++v) red[((i * TN + j) * 16 + v) * 64] = acc[i][j][v];
    }
    __syncthreads();
    if (kgrp == 0) {
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int v = 0; v < 16; ++v) acc[i][j][v] += red[((i * TN + j) * 16 + v) * 64];
    }
    __syncthreads();   // the output tile below overwrites what was just read
  }
  if (MODE == MODE_PLAIN) {   // fp32 rows straight from the accumulators: 32 consecutive columns per row and block
    float *out = static_cast<float *>(a.Out);
    if (kgrp == 0) {
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int mi = m0 + (wm * TM + i) * 32 + 8 * (v / 4) + 4 * (lane >> 5) + (v % 4);
            if (mi < a.M) out[size_t(mi) * a.N + n0 + (wn * TN + j) * 32 + (lane & 31)] = acc[i][j][v];
          }
    }
    return;
  }
  // ---- round once to bf16 into a row-major LDS tile ----
  // accumulator element v of lane L: row 8*(v/4) + 4*(L/32) + v%4, column L%32 of its 32x32 block
  uint16_t *sOut = reinterpret_cast<uint16_t *>(smem);   // [BM][BN] bf16
  if (kgrp == 0) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int row = (wm * TM + i) * 32 + 8 * (v / 4) + 4 * (lane >> 5) + (v % 4);
          const int col = (wn * TN + j) * 32 + (lane & 31);
          float val = acc[i][j][v];
          if (MODE == MODE_OPROJ) {   // the residual joins before the one rounding
            const long long ro = s_res[row];
            if (ro >= 0) val += to_float(static_cast<const bf16_t *>(a.Res)[ro + col]);
          }
          sOut[row * BN + col] = f32_to_bf16_rne(val);
        }
  }
  __syncthreads();
  // ---- scatter: every output row slice is contiguous in the cache; 16 bytes per lane ----
  bf16_t *dst_half = static_cast<bf16_t *>(MODE == MODE_OPROJ ? a.Out
                                           : MODE == MODE_QKV ? (section == 0 ? a.Out : section == 1 ? a.Kc : a.Vc)
                                                              : (section == 0 ? a.Kc : a.Vc));
  // Rotary embedding (query and key tiles, when the tile holds whole heads): the rounded row is turned by its
  // token's position on the way out, in fp32, and rounded again.  A thread takes 8 planes at a time: the 8-element
  // vectors of elements j and j + d/2 of a head, which share their angles; the angles of two such pairs are fetched
  // before either is used (a fetch costs a trip to the L2).
  const bool turn = (MODE == MODE_REBUILD ? section == 0 : MODE == MODE_QKV ? section <= 1 : false) && a.rope != nullptr;
  if (turn) {
    constexpr int PV = BM * BN / 16;           // pairs of vectors in the tile
    const int half = a.d / 2, hv = half / 8;   // vectors per half head
    const int per_row = BN / 16;
    for (int i0 = 0; i0 < (PV + 511) / 512; i0 += 2) {
      float2 cs[2][8];
      u32x4 lo[2], hi[2];
      long long offv[2];
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const int idx = tid + (i0 + u) * 512;
        offv[u] = -1;
        if (idx < PV) {
          const int row = idx / per_row, rem = idx - row * per_row;
          const int hh = rem / hv, v = rem - hh * hv;
          const long long off = s_dst[row * nh + hh];
          if (off >= 0) {
            offv[u] = off + v * 8;
            const float2 *src = a.rope + size_t(s_rpos[row]) * half + v * 8;
#pragma unroll
            for (int e = 0; e < 8; ++e) cs[u][e] = src[e];
            lo[u] = *reinterpret_cast<const u32x4 *>(sOut + row * BN + hh * a.d + v * 8);
            hi[u] = *reinterpret_cast<const u32x4 *>(sOut + row * BN + hh * a.d + half + v * 8);
          }
        }
      }
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        if (offv[u] < 0) continue;
        uint32_t rl[8], rh[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float x = __uint_as_float(((lo[u][e / 2] >> (16 * (e & 1))) & 0xffffu) << 16);
          const float y = __uint_as_float(((hi[u][e / 2] >> (16 * (e & 1))) & 0xffffu) << 16);
          rl[e] = f32_to_bf16_rne(rope_lo(x, y, cs[u][e]));
          rh[e] = f32_to_bf16_rne(rope_hi(x, y, cs[u][e]));
        }
        *reinterpret_cast<u32x4 *>(dst_half + offv[u]) =
            u32x4{rl[0] | (rl[1] << 16), rl[2] | (rl[3] << 16), rl[4] | (rl[5] << 16), rl[6] | (rl[7] << 16)};
        *reinterpret_cast<u32x4 *>(dst_half + offv[u] + half) =
            u32x4{rh[0] | (rh[1] << 16), rh[2] | (rh[3] << 16), rh[4] | (rh[5] << 16), rh[6] | (rh[7] << 16)};
      }
    }
    return;
  }
  constexpr int VPR = BN / 8;   // 16-byte vectors per tile row
  for (int idx = tid; idx < BM * VPR; idx += 512) {
    const int row = idx / VPR, vec = idx - row * VPR;
    const long long off = s_dst[row * nh + (vec * 8) / sw];
    if (off >= 0) {
      const u32x4 val = *reinterpret_cast<const u32x4 *>(sOut + row * BN + vec * 8);
      *reinterpret_cast<u32x4 *>(dst_half + off + (vec * 8) % sw) = val;
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
  if (pos < 0) return;   // an empty rank (uniform over the wave)
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
    if (slot < 0) return;   // the head still holds this token's row
    T *dst = static_cast<T *>(half ? a.Vc : a.Kc) + ((size_t(b) * a.H + h) * a.K + slot) * a.d + cc;
    store_elem(dst, s);
    if (a.map_dst && half == 0 && cc == 0) {
      a.map_dst[(size_t(b) * a.H + h) * a.K + slot] = pos;
      if (a.map_out) a.map_out[(size_t(b) * a.H + h) * a.K + slot] = pos;
    }
  }
}

// The forward's two projections (QKV, OPROJ) for storage types and widths the tile kernel does not take (fp32
// storage, widths that are no multiples of 128): one wave per output element, all r + 1 rows of a sequence alike
// (rank j < r, the current token at j = r).  fp32 products and sums, one rounding to the storage type.
template <typename T, int MODE>
__global__ __launch_bounds__(256) void proj_dot_kernel(const GemmArgs a) {
  constexpr int EPL = Vec16<T>::EPL;
  const size_t wid = (size_t(blockIdx.x) * blockDim.x + threadIdx.x) >> 6;
  const int lane = threadIdx.x & 63;
  const int rps = a.r + 1;
  if (wid >= size_t(a.B) * rps * a.N) return;
  const int mi = int(wid / a.N), nf = int(wid - size_t(mi) * a.N);
  const int b = mi / rps, j = mi - b * rps;
  const bool cur = j == a.r;
  const int pos = cur ? a.cur_pos : a.rebuilt_pos[size_t(b) * a.Rdim + j];
  if (pos < 0) return;   // an empty rank (uniform over the wave)
  const int Hd = a.H * a.d;
  const size_t xrow = a.a_gather ? size_t(b) * a.N_max + pos : size_t(b) * a.xrps + j;
  const T *x = static_cast<const T *>(a.X) + xrow * a.D;
  const T *wrow = MODE == MODE_QKV && nf < Hd ? static_cast<const T *>(a.Wq) + size_t(nf) * a.D
                  : MODE == MODE_QKV          ? static_cast<const T *>(a.W) + size_t(nf - Hd) * a.D
                                              : static_cast<const T *>(a.W) + size_t(nf) * a.D;
  float s = 0.f;
  for (int c = lane * EPL; c < a.D; c += 64 * EPL) {
    float xf[EPL], wf[EPL];
    Vec16<T>::load(x + c, xf);
    Vec16<T>::load(wrow + c, wf);
#pragma unroll
    for (int e = 0; e < EPL; ++e) s = fmaf(xf[e], wf[e], s);
  }
  s = wave_sum(s);
  if (lane != 0) return;
  if (MODE == MODE_OPROJ) {
    const size_t rrow = a.res_gather ? size_t(b) * a.N_max + pos : size_t(b) * a.xrps + j;
    s += to_float(static_cast<const T *>(a.Res)[rrow * a.N + nf]);
    store_elem(static_cast<T *>(a.Out) + (size_t(b) * a.out_rps + (cur ? a.out_cur : j)) * a.N + nf, s);
    return;
  }
  const int section = nf / Hd, rem = nf - section * Hd;
  if (section == 0) {
    store_elem(static_cast<T *>(a.Out) + (size_t(b) * a.xrps + j) * Hd + rem, s);
    return;
  }
  const int h = rem / a.d, cc = rem - h * a.d;
  const int slot = cur ? a.insert_slot[size_t(b) * a.H + h] : a.free_list[(size_t(b) * a.H + h) * a.R1 + j];
  store_elem(static_cast<T *>(section == 1 ? a.Kc : a.Vc) + ((size_t(b) * a.H + h) * a.K + slot) * a.d + cc, s);
}

// The current token's row of every sequence (rebuild forward): B rows against the same weights, a skinny product
// that only streams W.  One workgroup owns 16 sequences x NC*16 output columns; its 4 waves cut the contraction
// into quarters (summed through LDS in a fixed order).  16x16x32 tiles; lane (c, g) holds, for matrix instruction
// s, the 8 values at k = (4*s + g)*8 of its quarter for row c, so every row is read in 64-byte runs (both operands
// use the same assignment, so the order of k does not matter).  Epilogue as in the tile kernel.
template <int MODE, int NC>
__global__ __launch_bounds__(256) void cur_rows_kernel(const GemmArgs a) {
  typedef float f32x4 __attribute__((ext_vector_type(4)));
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int c = lane & 15, g = lane >> 4;
  const int j0 = blockIdx.x * (16 * NC), t0 = blockIdx.y * 16;
  const int Hd = a.H * a.d;
  const int kw = a.D / 4;                               // k-range of one wave, a multiple of 32
  const int bb = min(t0 + c, a.B - 1);                  // padded rows read a valid sequence; dropped at the store
  const size_t xrow = a.a_gather ? size_t(bb) * a.N_max + a.cur_pos : size_t(bb) * a.xrps + a.r;
  const u32x4 *pa = reinterpret_cast<const u32x4 *>(static_cast<const bf16_t *>(a.X) + xrow * a.D + wave * kw) + g;
  const u32x4 *pb[NC];
#pragma unroll
  for (int nc = 0; nc < NC; ++nc) {
    const int n = j0 + nc * 16 + c;                     // N is a multiple of 16 * NC
    const bf16_t *wrow = MODE == MODE_QKV && n < Hd ? static_cast<const bf16_t *>(a.Wq) + size_t(n) * a.D
                         : MODE == MODE_QKV         ? static_cast<const bf16_t *>(a.W) + size_t(n - Hd) * a.D
                                                    : static_cast<const bf16_t *>(a.W) + size_t(n) * a.D;
    pb[nc] = reinterpret_cast<const u32x4 *>(wrow + wave * kw) + g;
  }
  f32x4 acc[NC];
#pragma unroll
  for (int nc = 0; nc < NC; ++nc) acc[nc] = f32x4{0.f, 0.f, 0.f, 0.f};
  const int steps = kw / 32;
#define CUR_STEP(VA, VB)                                                                                     \
  _Pragma("unroll") for (int nc = 0; nc < NC; ++nc)                                                          \
    acc[nc] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*reinterpret_cast<const bf16x8 *>(&(VA)),              \
                                                      *reinterpret_cast<const bf16x8 *>(&(VB)[nc]), acc[nc], 0, 0, 0);
  int s = 0;
  for (; s + 4 <= steps; s += 4) {          // four steps' loads in flight
    u32x4 va[4], vb[4][NC];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      va[u] = pa[(s + u) * 4];
#pragma unroll
      for (int nc = 0; nc < NC; ++nc) vb[u][nc] = pb[nc][(s + u) * 4];
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) { CUR_STEP(va[u], vb[u]) }
  }
  for (; s < steps; ++s) {
    u32x4 va = pa[s * 4], vb[NC];
#pragma unroll
    for (int nc = 0; nc < NC; ++nc) vb[nc] = pb[nc][s * 4];
    CUR_STEP(va, vb)
  }
#undef CUR_STEP
  // accumulator element v of lane (c, g): sequence 4*g + v, column c
  __shared__ float red[4][NC][16][17];
#pragma unroll
  for (int nc = 0; nc < NC; ++nc)
#pragma unroll
    for (int v = 0; v < 4; ++v) red[wave][nc][4 * g + v][c] = acc[nc][v];
  __syncthreads();
  const int m = tid >> 4, nn = tid & 15;
  const int b = t0 + m;
  if (b >= a.B) return;
#pragma unroll
  for (int nc = 0; nc < NC; ++nc) {
    float val = (red[0][nc][m][nn] + red[1][nc][m][nn]) + (red[2][nc][m][nn] + red[3][nc][m][nn]);
    const int n = j0 + nc * 16 + nn;
    bf16_t *dst;
    if (MODE == MODE_OPROJ) {
      const size_t rrow = a.res_gather ? size_t(b) * a.N_max + a.cur_pos : size_t(b) * a.xrps + a.r;
      val += to_float(static_cast<const bf16_t *>(a.Res)[rrow * a.N + n]);
      dst = static_cast<bf16_t *>(a.Out) + (size_t(b) * a.out_rps + a.out_cur) * a.N + n;
    } else {
      const int section = n / Hd, rem = n - section * Hd;
      const int h = rem / a.d;
      if (section == 0) {
        dst = static_cast<bf16_t *>(a.Out) + (size_t(b) * a.xrps + a.r) * Hd + rem;
      } else {
        const int slot = a.insert_slot[size_t(b) * a.H + h];
        dst = static_cast<bf16_t *>(section == 1 ? a.Kc : a.Vc) + ((size_t(b) * a.H + h) * a.K + slot) * a.d + (rem - h * a.d);
      }
    }
    dst->bits = f32_to_bf16_rne(val);
  }
}

// The tile shapes the launcher chooses from, largest first.
struct TileShape {
  int bm, bn, bk;
};
constexpr TileShape kTiles[] = {{256, 256, 32}, {256, 128, 64}, {128, 128, 64}, {128, 64, 64}, {128, 32, 64}};
constexpr int kNumTiles = sizeof(kTiles) / sizeof(kTiles[0]);

// kdim = length of the contraction; scatter modes write head slices (section = H*d columns of one kind)
bool tile_fits(const TileShape &t, int kdim, int section, int head_dim, bool dense) {
  if (kdim % t.bk != 0 || section % t.bn != 0) return false;
  return dense || t.bn % head_dim == 0 || head_dim % t.bn == 0;
}

// Time of one workgroup on its tile in microseconds at a contraction length of 4096, measured with one tile per
// compute unit (largest tile first); the launch takes ceil(tiles / 256) rounds of that.  The tile with the lowest
// estimate is used: a launch that fills three quarters of the units once (256x128 at M = 512, N = 12288: 192 tiles,
// 64 us) beats one that fills all of them one and a half times (128x128: 384 tiles, 88 us).
constexpr float kTileMicros[kNumTiles] = {125.f, 66.f, 41.f, 40.f, 25.f};

// extra: workgroups that ride in the launch and need a compute unit each (the current tokens' rows)
int pick_tile(int M, int N, int kdim, int section, int head_dim, bool dense, int extra = 0) {
  int pick = -1;
  float best = 0.f;
  for (int i = 0; i < kNumTiles; ++i) {
    if (!tile_fits(kTiles[i], kdim, section, head_dim, dense)) continue;
    const long long tiles = (long long)((M + kTiles[i].bm - 1) / kTiles[i].bm) * (N / kTiles[i].bn);
    const float est = float((tiles + extra + 255) / 256) * kTileMicros[i];
    if (pick < 0 || est < best) {
      pick = i;
      best = est;
    }
  }
  if (const char *e = getenv("ADORE_GEMM_TILE")) {   // tuning runs: force a tile shape by index
    const int v = atoi(e);
    if (v >= 0 && v < kNumTiles && tile_fits(kTiles[v], kdim, section, head_dim, dense)) pick = v;
  }
  return pick;
}

template <int MODE>
void launch_tile(ScopedTimer &t, hipStream_t stream, int pick, GemmArgs &a) {
  a.tiles_m = (a.M + kTiles[pick].bm - 1) / kTiles[pick].bm;
  a.tiles_n = a.N / kTiles[pick].bn;
  const int total = a.tiles_m * a.tiles_n;
  const dim3 grid((total + 7) / 8 * 8 + a.n_cur), block(512);
  //                                              BM   BN  BK KG WM WN LS NS
  switch (pick) {
    case 0: ADORE_LAUNCH(t, (rebuild_mfma_kernel<MODE, 256, 256, 32, 1, 2, 4, 4, 2>), grid, block, 0, stream, a); break;
    case 1: ADORE_LAUNCH(t, (rebuild_mfma_kernel<MODE, 256, 128, 64, 1, 4, 2, 3, 2>), grid, block, 0, stream, a); break;
    case 2: ADORE_LAUNCH(t, (rebuild_mfma_kernel<MODE, 128, 128, 64, 2, 2, 2, 3, 4>), grid, block, 0, stream, a); break;
    case 3: ADORE_LAUNCH(t, (rebuild_mfma_kernel<MODE, 128, 64, 64, 2, 2, 2, 3, 4>), grid, block, 0, stream, a); break;
    default: ADORE_LAUNCH(t, (rebuild_mfma_kernel<MODE, 128, 32, 64, 2, 4, 1, 3, 4>), grid, block, 0, stream, a); break;
  }
}

void fill_common(adore_ctx *ctx, GemmArgs &a, int lists, int r) {
  const adore_config &c = ctx->cfg;
  a.Wq = nullptr; a.Out = nullptr; a.Res = nullptr; a.map_dst = a.map_out = nullptr;
  a.rebuilt_pos = ctx->rebuilt_pos[lists];
  a.free_list = ctx->free_list[lists];
  a.insert_slot = ctx->insert_slot[lists];
  a.B = c.batch; a.H = c.heads; a.d = c.head_dim; a.D = c.hidden; a.K = c.cache_slots;
  a.N_max = c.max_positions; a.r = r; a.R1 = c.rebuild_budget + 1; a.Rdim = max(c.rebuild_budget, 1);
  a.xrps = r; a.cur_pos = 0; a.a_gather = 1; a.res_gather = 0; a.out_rps = 0; a.out_cur = 0;
  a.tiles_m = a.tiles_n = 0;
  a.n_cur = 0;
  a.cur_ks = 1;
  a.rope = nullptr;
  a.rope_cur = nullptr;
}

}  // namespace

hipError_t launch_rebuild_gemm(adore_ctx *ctx, int layer, const void *hidden_layer, int lists, int r,
                               int32_t *map_dst, int32_t *map_out) {
  const adore_config &c = ctx->cfg;
  if (r <= 0) return hipSuccess;
  const size_t es = elem_size(c);
  const size_t layer_bytes = size_t(c.batch) * c.heads * c.cache_slots * c.head_dim * es;
  GemmArgs a;
  fill_common(ctx, a, lists, r);
  a.X = hidden_layer;
  a.W = static_cast<const char *>(ctx->w.w_kv) + size_t(layer) * 2 * c.heads * c.head_dim * c.hidden * es;
  a.Kc = ctx->cache_k + layer * layer_bytes;
  a.Vc = ctx->cache_v + layer * layer_bytes;
  a.M = c.batch * r; a.N = 2 * c.heads * c.head_dim;
  a.map_dst = map_dst; a.map_out = map_out;
  ScopedTimer t(ctx, ADORE_KERNEL_REBUILD_GEMM, ctx->stream);
  const int pick = c.dtype == ADORE_BF16 ? pick_tile(a.M, a.N, c.hidden, c.heads * c.head_dim, c.head_dim, false) : -1;
  // the key tiles turn their rows themselves when a tile holds whole heads; otherwise a pass of its own follows
  const bool rope = c.rope_base > 0.f;
  const bool turned = rope && pick >= 0 && kTiles[pick].bn >= c.head_dim;
  if (turned) a.rope = ctx->rope_f;
  if (pick >= 0) {
    launch_tile<MODE_REBUILD>(t, ctx->stream, pick, a);
  } else {
    const size_t waves = size_t(a.M) * a.N;
    const unsigned blocks = unsigned((waves + 3) / 4);
    if (c.dtype == ADORE_BF16) {
      ADORE_LAUNCH(t, (rebuild_dot_kernel<bf16_t>), dim3(blocks), dim3(256), 0, ctx->stream, a);
    } else {
      ADORE_LAUNCH(t, (rebuild_dot_kernel<float>), dim3(blocks), dim3(256), 0, ctx->stream, a);
    }
  }
  hipError_t e = hipGetLastError();
  if (e == hipSuccess && rope && !turned) e = launch_rope_rows(ctx, layer, lists, r, 0, r, false, 0);
  return e;
}

// ---- rebuild forward: the two projections around the attention of a layer ----------------------------
// Whether the tile kernels take both projections of this configuration; otherwise the forward runs them as one
// wave per output element (proj_dot_kernel).
bool fwd_gemm_supported(const adore_config &c) {
  const int Hd = c.heads * c.head_dim;
  return c.dtype == ADORE_BF16 && c.hidden % 128 == 0 && Hd % 128 == 0 &&
         pick_tile(1, 3 * Hd, c.hidden, Hd, c.head_dim, false) >= 0 &&
         pick_tile(1, c.hidden, Hd, c.hidden, c.head_dim, true) >= 0;
}

namespace {

// Workgroups that take the current tokens' rows inside the tile launch (a multiple of 8; see cur_rows_role) when
// the contraction is cut ks ways inside a workgroup, or 0 when the rows go through a launch of their own: a
// width that is no multiple of the role's 256 columns, or ADORE_FWD_CUR_SEPARATE=1 (for comparison runs).
int cur_row_riders(const GemmArgs &a, int ks) {
  if (a.N % kCurCols != 0 || a.D % (64 * ks) != 0) return 0;
  if (const char *e = getenv("ADORE_FWD_CUR_SEPARATE")) {
    if (atoi(e) != 0) return 0;
  }
  const int n = ((a.B + 15) / 16) * (a.N / (kCurCols / ks));
  return (n + 7) / 8 * 8;
}

// Tile shape and cut for a forward projection: the cheapest launch by pick_tile's estimate, with the rows of the
// current tokens spread over as many of the remaining units as a cut of the contraction allows.
int pick_with_riders(GemmArgs &a, int kdim, int section, int head_dim, bool dense) {
  a.n_cur = 0;
  a.cur_ks = 1;
  const int base = cur_row_riders(a, 1);
  const int pick = pick_tile(a.M, a.N, kdim, section, head_dim, dense, base);
  if (pick < 0 || base == 0) return pick;
  const int tiles = ((a.M + kTiles[pick].bm - 1) / kTiles[pick].bm) * (a.N / kTiles[pick].bn);
  const int rounds = (tiles + base + 255) / 256;
  int ks = 1;
  while (ks < 8 && cur_row_riders(a, ks * 2) > 0 && (tiles + cur_row_riders(a, ks * 2) + 255) / 256 <= rounds) ks *= 2;
  a.cur_ks = ks;
  a.n_cur = cur_row_riders(a, ks);
  return pick;
}

template <int MODE>
void launch_proj_dot(ScopedTimer &t, hipStream_t stream, bool bf16, const GemmArgs &a) {
  const size_t waves = size_t(a.B) * (a.r + 1) * a.N;
  const dim3 grid(unsigned((waves + 3) / 4)), block(256);
  if (bf16) {
    ADORE_LAUNCH(t, (proj_dot_kernel<bf16_t, MODE>), grid, block, 0, stream, a);
  } else {
    ADORE_LAUNCH(t, (proj_dot_kernel<float, MODE>), grid, block, 0, stream, a);
  }
}

template <int MODE>
void launch_cur_rows(ScopedTimer &t, hipStream_t stream, const GemmArgs &a) {
  const int seq_blocks = (a.B + 15) / 16;
  if (a.N % 32 == 0 && (a.N / 32) * seq_blocks >= 256) {
    ADORE_LAUNCH(t, (cur_rows_kernel<MODE, 2>), dim3(a.N / 32, seq_blocks), dim3(256), 0, stream, a);
  } else {
    ADORE_LAUNCH(t, (cur_rows_kernel<MODE, 1>), dim3(a.N / 16, seq_blocks), dim3(256), 0, stream, a);
  }
}

}  // namespace

// q, k, v of the r rebuilt tokens and the current token of every sequence.  x_rows: the rows entering this layer,
// either the embedding table [B][N_max][D] (by_position) or the dense rows [B][r+1][D] the previous layer wrote.
hipError_t launch_fwd_qkv(adore_ctx *ctx, int layer, const void *w_q_layer, const void *x_rows, bool by_position,
                          int r) {
  const adore_config &c = ctx->cfg;
  const int Hd = c.heads * c.head_dim;
  const size_t es = elem_size(c);
  const size_t layer_bytes = size_t(c.batch) * Hd * c.cache_slots * es;
  GemmArgs a;
  fill_common(ctx, a, ctx->cur, r);
  a.X = x_rows;
  a.W = static_cast<const char *>(ctx->w.w_kv) + size_t(layer) * 2 * Hd * c.hidden * es;
  a.Wq = w_q_layer;
  a.Kc = ctx->cache_k + layer * layer_bytes;
  a.Vc = ctx->cache_v + layer * layer_bytes;
  a.Out = ctx->fwd_q;
  a.xrps = r + 1; a.cur_pos = ctx->n; a.a_gather = by_position ? 1 : 0;
  a.M = c.batch * r; a.N = 3 * Hd;
  bool turned = false;   // the tiles turned the rebuilt tokens' query and key rows themselves
  bool cur_turned = false;   // ... and the workgroups of the current tokens' rows theirs
  if (!fwd_gemm_supported(c)) {   // all r + 1 rows of every sequence, one wave per output element
    {
      ScopedTimer t(ctx, ADORE_KERNEL_FWD_QKV, ctx->stream);
      launch_proj_dot<MODE_QKV>(t, ctx->stream, c.dtype == ADORE_BF16, a);
    }
    hipError_t e = hipGetLastError();
    if (e == hipSuccess) e = launch_rope_rows(ctx, layer, ctx->cur, r, 0, r + 1, true, ctx->n);
    return e;
  }
  if (r > 0) {
    ScopedTimer t(ctx, ADORE_KERNEL_FWD_QKV, ctx->stream);
    const int pick = pick_with_riders(a, c.hidden, Hd, c.head_dim, false);
    if (pick < 0) return hipErrorInvalidValue;
    turned = c.rope_base > 0.f && kTiles[pick].bn >= c.head_dim;
    if (turned) a.rope = ctx->rope_f;
    // the current tokens' rows riding in this launch turn themselves when a workgroup's columns are whole heads
    cur_turned = c.rope_base > 0.f && a.n_cur > 0 && (kCurCols / a.cur_ks) % c.head_dim == 0;
    if (cur_turned) a.rope_cur = ctx->rope_f;
    launch_tile<MODE_QKV>(t, ctx->stream, pick, a);
  }
  if (a.n_cur == 0) {
    ScopedTimer t(ctx, ADORE_KERNEL_FWD_QKV_CUR, ctx->stream);
    launch_cur_rows<MODE_QKV>(t, ctx->stream, a);
  }
  hipError_t e = hipGetLastError();
  // rotary embedding: whatever rows the launch above did not turn itself
  if (e == hipSuccess) e = launch_rope_rows(ctx, layer, ctx->cur, r, turned ? r : 0, cur_turned ? r : r + 1, true, ctx->n);
  return e;
}

// x' = round(x + W_o . o): residual rows like launch_fwd_qkv's x_rows; output rows at out[b * out_rps + j] for
// rank j and out[b * out_rps + out_cur] for the current token.
hipError_t launch_fwd_oproj(adore_ctx *ctx, const void *w_o_layer, const void *x_rows, bool by_position, void *out,
                            int out_rps, int out_cur, int r) {
  const adore_config &c = ctx->cfg;
  const int Hd = c.heads * c.head_dim;
  GemmArgs a;
  fill_common(ctx, a, ctx->cur, r);
  a.X = ctx->fwd_o;
  a.W = w_o_layer;
  a.Kc = a.Vc = nullptr;
  a.Out = out;
  a.Res = x_rows;
  a.D = Hd;
  a.xrps = r + 1; a.cur_pos = ctx->n; a.a_gather = 0; a.res_gather = by_position ? 1 : 0;
  a.out_rps = out_rps; a.out_cur = out_cur;
  a.M = c.batch * r; a.N = c.hidden;
  if (!fwd_gemm_supported(c)) {
    ScopedTimer t(ctx, ADORE_KERNEL_FWD_OPROJ, ctx->stream);
    launch_proj_dot<MODE_OPROJ>(t, ctx->stream, c.dtype == ADORE_BF16, a);
    return hipGetLastError();
  }
  if (r > 0) {
    ScopedTimer t(ctx, ADORE_KERNEL_FWD_OPROJ, ctx->stream);
    const int pick = pick_with_riders(a, Hd, c.hidden, c.head_dim, true);
    if (pick < 0) return hipErrorInvalidValue;
    launch_tile<MODE_OPROJ>(t, ctx->stream, pick, a);
  }
  if (a.n_cur == 0) {
    ScopedTimer t(ctx, ADORE_KERNEL_FWD_OPROJ_CUR, ctx->stream);
    launch_cur_rows<MODE_OPROJ>(t, ctx->stream, a);
  }
  return hipGetLastError();
}
// gi[tok][j] = W_ih[j][:] . x_tok for the ntok tokens of a prompt chunk (token b * per_seq + i at row
// b * seq_rows + i of x), fp32, on the 128x128 tile.  False if the shape does not fit that tile.
bool launch_plain_projection(adore_ctx *ctx, ScopedTimer &t, hipStream_t st, const void *x, const void *W, float *out,
                             int ntok, int per_seq, int seq_rows, int N, int D) {
  constexpr int kTile = 2;   // 128 x 128 x 64
  if (ctx->cfg.dtype != ADORE_BF16 || N % kTiles[kTile].bn != 0 || D % kTiles[kTile].bk != 0) return false;
  GemmArgs a;
  fill_common(ctx, a, 0, per_seq);
  a.X = x; a.W = W; a.Out = out;
  a.Kc = a.Vc = nullptr;
  a.D = D; a.M = ntok; a.N = N;
  a.xrps = seq_rows; a.a_gather = 0;
  a.tiles_m = (a.M + kTiles[kTile].bm - 1) / kTiles[kTile].bm;
  a.tiles_n = a.N / kTiles[kTile].bn;
  const dim3 grid((a.tiles_m * a.tiles_n + 7) / 8 * 8), block(512);
  ADORE_LAUNCH(t, (rebuild_mfma_kernel<MODE_PLAIN, 128, 128, 64, 2, 2, 2, 3, 4>), grid, block, 0, st, a);
  return true;
}

}  // namespace adore
