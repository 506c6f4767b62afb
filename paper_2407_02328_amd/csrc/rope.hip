// Rotary position embedding of the rows a projection has just written (optional, adore_config::rope_base > 0).
//
// The backbones the paper evaluates turn every query and key by its token's position before the product
// (the paper names the embedding in its related work on length extrapolation).  A key that is rebuilt from a
// hidden state (Sec. 2.3) therefore has to be turned to the position its token had.  As in those models the
// projection leaves the matrix product in the storage type; elements j and j + d/2 of a head are then turned by
// the angle pos * base^(-2j/d) and rounded again:
//
//   out[j]       = x[j] cos t - x[j + d/2] sin t
//   out[j + d/2] = x[j] sin t + x[j + d/2] cos t
//
// The table of (cos, sin) per (position, j) is made once per init in fp64, with a copy rounded to fp32 behind it.
// fp32 storage: the rotation runs in fp64, so the result is the correctly rounded rotation of what the projection
// stored.  bf16 storage: fp32 (fused multiply-add), the same expression wherever a row is turned (here and in the
// tile kernel's epilogue).  One thread per pair; the rows are found through the same lists the projection
// scattered by.
#include "adore_internal.h"
#include "device_utils.h"

namespace adore {

namespace {

__global__ __launch_bounds__(256) void rope_table_kernel(double2 *tab, float2 *tab_f, int n_pos, int half, double base) {
  const size_t idx = size_t(blockIdx.x) * 256 + threadIdx.x;
  if (idx >= size_t(n_pos) * half) return;
  const int pos = int(idx / half), j = int(idx - size_t(pos) * half);
  const double t = double(pos) * pow(base, -double(j) / double(half));   // base^(-2j/d)
  double s, c;
  sincos(t, &s, &c);
  tab[idx] = double2{c, s};
  tab_f[idx] = float2{float(c), float(s)};
}

__device__ inline void turn_plane(float *lo_p, float *hi_p, const double2 *tab, const float2 *, size_t at) {
  const double2 cs = tab[at];
  const double lo = double(*lo_p), hi = double(*hi_p);
  *lo_p = float(rope_lo(lo, hi, cs));
  *hi_p = float(rope_hi(lo, hi, cs));
}
__device__ inline void turn_plane(bf16_t *lo_p, bf16_t *hi_p, const double2 *, const float2 *tab_f, size_t at) {
  const float2 cs = tab_f[at];
  const float lo = to_float(*lo_p), hi = to_float(*hi_p);
  lo_p->bits = f32_to_bf16_rne(rope_lo(lo, hi, cs));
  hi_p->bits = f32_to_bf16_rne(rope_hi(lo, hi, cs));
}

struct RopeArgs {
  void *Kc;                    // [B][H][K][d] of this layer
  void *Q;                     // forward: query rows [B * xrps][H*d], or null
  const double2 *tab;          // [N_max][d/2] (cos, sin)
  const float2 *tab_f;         // the same rounded to fp32
  const int32_t *rebuilt_pos;  // [B][Rdim]
  const int32_t *free_list;    // [B][H][R1]   slot of rank j
  const int32_t *insert_slot;  // [B][H]       forward: slot of the current token
  int B, H, d, K, r, R1, Rdim, xrps, cur_pos;
  int j0, rows;                // rows j0 .. j0 + rows - 1 of every (b, h); row r is the current token (forward)
};

// thread -> (kind: key row / query row, b, h, row j, pair)
template <typename T>
__global__ __launch_bounds__(256) void rope_rows_kernel(const RopeArgs a) {
  const int half = a.d / 2;
  const size_t per_kind = size_t(a.B) * a.H * a.rows * half;
  size_t idx = size_t(blockIdx.x) * 256 + threadIdx.x;
  const bool query = idx >= per_kind;
  if (query) {
    idx -= per_kind;
    if (!a.Q || idx >= per_kind) return;
  }
  const int jp = int(idx % half);
  size_t t = idx / half;
  const int j = a.j0 + int(t % a.rows);
  t /= a.rows;
  const int h = int(t % a.H), b = int(t / a.H);
  const bool cur = j >= a.r;
  const int pos = cur ? a.cur_pos : a.rebuilt_pos[size_t(b) * a.Rdim + j];
  T *row;
  if (query) {
    row = static_cast<T *>(a.Q) + (size_t(b) * a.xrps + j) * a.H * a.d + size_t(h) * a.d;
  } else {
    const int slot = cur ? a.insert_slot[size_t(b) * a.H + h] : a.free_list[(size_t(b) * a.H + h) * a.R1 + j];
    row = static_cast<T *>(a.Kc) + ((size_t(b) * a.H + h) * a.K + slot) * a.d;
  }
  turn_plane(row + jp, row + jp + half, a.tab, a.tab_f, size_t(pos) * half + jp);
}

hipError_t launch_rows(adore_ctx *ctx, const RopeArgs &a) {
  const size_t threads = size_t(a.B) * a.H * a.rows * (a.d / 2) * (a.Q ? 2 : 1);
  if (threads == 0) return hipSuccess;
  ScopedTimer t(ctx, ADORE_KERNEL_ROPE, ctx->stream);
  const dim3 grid(unsigned((threads + 255) / 256)), block(256);
  if (ctx->cfg.dtype == ADORE_BF16) {
    ADORE_LAUNCH(t, (rope_rows_kernel<bf16_t>), grid, block, 0, ctx->stream, a);
  } else {
    ADORE_LAUNCH(t, (rope_rows_kernel<float>), grid, block, 0, ctx->stream, a);
  }
  return hipGetLastError();
}

}  // namespace

hipError_t launch_rope_table(adore_ctx *ctx) {
  const adore_config &c = ctx->cfg;
  if (!(c.rope_base > 0.f)) return hipSuccess;
  const int half = c.head_dim / 2;
  const size_t n = size_t(c.max_positions) * half;
  hipLaunchKernelGGL(rope_table_kernel, dim3(unsigned((n + 255) / 256)), dim3(256), 0, ctx->stream,
                     static_cast<double2 *>(ctx->rope), ctx->rope_f, c.max_positions, half, double(c.rope_base));
  return hipGetLastError();
}

// Rows j0 .. j1-1 of every (sequence, head) of `layer`: rank j < r is a rebuilt token (its slot and position from
// ring copy `lists`), j = r the current token at position cur_pos (forward).  queries: the rows of the forward's
// query buffer as well.
hipError_t launch_rope_rows(adore_ctx *ctx, int layer, int lists, int r, int j0, int j1, bool queries, int cur_pos) {
  const adore_config &c = ctx->cfg;
  if (!(c.rope_base > 0.f) || j1 <= j0) return hipSuccess;
  const size_t layer_bytes = size_t(c.batch) * c.heads * c.cache_slots * c.head_dim * elem_size(c);
  RopeArgs a;
  a.Kc = ctx->cache_k + layer * layer_bytes;
  a.Q = queries ? ctx->fwd_q : nullptr;
  a.tab = static_cast<const double2 *>(ctx->rope);
  a.tab_f = ctx->rope_f;
  a.rebuilt_pos = ctx->rebuilt_pos[lists];
  a.free_list = ctx->free_list[lists];
  a.insert_slot = ctx->insert_slot[lists];
  a.B = c.batch; a.H = c.heads; a.d = c.head_dim; a.K = c.cache_slots;
  a.r = r; a.R1 = c.rebuild_budget + 1; a.Rdim = max(c.rebuild_budget, 1);
  a.xrps = r + 1; a.cur_pos = cur_pos; a.j0 = j0; a.rows = j1 - j0;
  return launch_rows(ctx, a);
}

}  // namespace adore
