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
// The table of (cos, sin) per (position, j) is made once per init in fp64 and the rotation itself runs in fp64:
// a few flops per element on a few MB, so that the result is the correctly rounded rotation of what the
// projection stored.  One thread per pair; the rows are found through the same lists the projection scattered by.
#include "adore_internal.h"
#include "device_utils.h"

namespace adore {

namespace {

__global__ __launch_bounds__(256) void rope_table_kernel(double2 *tab, int n_pos, int half, double base) {
  const size_t idx = size_t(blockIdx.x) * 256 + threadIdx.x;
  if (idx >= size_t(n_pos) * half) return;
  const int pos = int(idx / half), j = int(idx - size_t(pos) * half);
  const double t = double(pos) * pow(base, -double(j) / double(half));   // base^(-2j/d)
  double s, c;
  sincos(t, &s, &c);
  tab[idx] = double2{c, s};
}

// One rounding from fp64 to bf16: through fp32, stepping off a bf16 midpoint that only the first rounding produced.
__device__ inline uint16_t f64_to_bf16_rne(double v) {
  const float f = float(v);
  uint32_t u = __float_as_uint(f);
  if ((u & 0xffffu) == 0x8000u) {
    const double back = double(f);
    if (v != back) u = fabs(v) > fabs(back) ? u + 1u : u - 1u;
  }
  return f32_to_bf16_rne(__uint_as_float(u));
}

__device__ inline void store_f64(float *p, double v) { *p = float(v); }
__device__ inline void store_f64(bf16_t *p, double v) { p->bits = f64_to_bf16_rne(v); }

struct RopeArgs {
  void *Kc;                    // [B][H][K][d] of this layer
  void *Q;                     // forward: query rows [B * xrps][H*d], or null
  const double2 *tab;          // [N_max][d/2] (cos, sin)
  const int32_t *rebuilt_pos;  // [B][Rdim]
  const int32_t *free_list;    // [B][H][R1]   slot of rank j
  const int32_t *insert_slot;  // [B][H]       forward: slot of the current token
  int B, H, d, K, r, R1, Rdim, xrps, cur_pos;
  int rows;                    // rows per (b, h): r, or r + 1 with the current token (forward)
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
  const int j = int(t % a.rows);
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
  const double2 cs = a.tab[size_t(pos) * half + jp];
  const double lo = double(to_float(row[jp])), hi = double(to_float(row[jp + half]));
  store_f64(row + jp, lo * cs.x - hi * cs.y);
  store_f64(row + jp + half, lo * cs.y + hi * cs.x);
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

RopeArgs common_args(adore_ctx *ctx, int layer, int lists, int r) {
  const adore_config &c = ctx->cfg;
  const size_t layer_bytes = size_t(c.batch) * c.heads * c.cache_slots * c.head_dim * elem_size(c);
  RopeArgs a;
  a.Kc = ctx->cache_k + layer * layer_bytes;
  a.Q = nullptr;
  a.tab = static_cast<const double2 *>(ctx->rope);
  a.rebuilt_pos = ctx->rebuilt_pos[lists];
  a.free_list = ctx->free_list[lists];
  a.insert_slot = ctx->insert_slot[lists];
  a.B = c.batch; a.H = c.heads; a.d = c.head_dim; a.K = c.cache_slots;
  a.r = r; a.R1 = c.rebuild_budget + 1; a.Rdim = max(c.rebuild_budget, 1);
  a.xrps = r + 1; a.cur_pos = 0; a.rows = r;
  return a;
}

}  // namespace

hipError_t launch_rope_table(adore_ctx *ctx) {
  const adore_config &c = ctx->cfg;
  if (!(c.rope_base > 0.f)) return hipSuccess;
  const int half = c.head_dim / 2;
  const size_t n = size_t(c.max_positions) * half;
  hipLaunchKernelGGL(rope_table_kernel, dim3(unsigned((n + 255) / 256)), dim3(256), 0, ctx->stream,
                     static_cast<double2 *>(ctx->rope), c.max_positions, half, double(c.rope_base));
  return hipGetLastError();
}

// Keys of the r tokens the rebuild projection of `layer` has just written (lists: ring copy of the step's lists).
hipError_t launch_rope_rebuilt(adore_ctx *ctx, int layer, int lists, int r) {
  if (!(ctx->cfg.rope_base > 0.f) || r <= 0) return hipSuccess;
  return launch_rows(ctx, common_args(ctx, layer, lists, r));
}

// Rebuild forward: keys and queries of the r rebuilt tokens and of the current token of every sequence.
hipError_t launch_rope_forward(adore_ctx *ctx, int layer, int r) {
  if (!(ctx->cfg.rope_base > 0.f)) return hipSuccess;
  RopeArgs a = common_args(ctx, layer, ctx->cur, r);
  a.Q = ctx->fwd_q;
  a.cur_pos = ctx->n;
  a.rows = r + 1;
  return launch_rows(ctx, a);
}

}  // namespace adore
