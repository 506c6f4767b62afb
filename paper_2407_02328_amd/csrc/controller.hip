// Stage 2: the controller module (paper Sec. 2.2, Eq. 2; App. "Implementation
// Details": GRU input size D -> d', position layer 1 -> d', interaction layer
// d' -> d' with tanh, output layer d' -> 1 with sigmoid).
//
//   z_i     = GRU(x_i, z_{i-1})
//   sigma_i = sigmoid(out_w . tanh(W_1 (p_i + z_i) + b_1) + out_b),  p_i = pos_w * (i * pos_scale) + pos_b
//
// Two kernels.  ctrl_input computes the input pre-activations W_ih x for a
// batch of tokens (the only part that reads D-wide data; it has no dependence
// between tokens, so a whole prompt chunk goes in one launch).  ctrl_cell does
// the recurrent part token by token: W_hh z, the gates, the MLP and the score.
// All sums are fp32 in a fixed order, so results are reproducible run to run.
#include "device_utils.h"

namespace adore {

namespace {

constexpr int JT = 4;  // gate rows per workgroup
constexpr int NB = 8;  // tokens per workgroup

// gi[tok][j] = sum_t W_ih[j][t] * x_tok[t]       (bias added in the cell kernel)
// Token tok = b * per_seq + i reads the row x[(b * seq_rows + i) * D].
template <typename T>
__global__ __launch_bounds__(256) void ctrl_input_kernel(const T *__restrict__ W_ih, const T *__restrict__ x,
                                                         float *__restrict__ gi, int D, int G3, int ntok,
                                                         int per_seq, int seq_rows) {
  constexpr int EPL = Vec16<T>::EPL;
  const int j0 = blockIdx.x * JT;
  const int t0 = blockIdx.y * NB;
  const int tid = threadIdx.x;
  float acc[JT][NB];
#pragma unroll
  for (int jj = 0; jj < JT; ++jj)
#pragma unroll
    for (int tt = 0; tt < NB; ++tt) acc[jj][tt] = 0.f;

  for (int c = tid * EPL; c < D; c += 256 * EPL) {
    float wf[JT][EPL];
#pragma unroll
    for (int jj = 0; jj < JT; ++jj) {
      if (j0 + jj < G3) {
        Vec16<T>::load(W_ih + size_t(j0 + jj) * D + c, wf[jj]);
      } else {
#pragma unroll
        for (int e = 0; e < EPL; ++e) wf[jj][e] = 0.f;
      }
    }
#pragma unroll
    for (int tt = 0; tt < NB; ++tt) {
      if (t0 + tt < ntok) {
        float xf[EPL];
        const int tok = t0 + tt;
        const size_t row = size_t(tok / per_seq) * seq_rows + tok % per_seq;
        Vec16<T>::load(x + row * D + c, xf);
#pragma unroll
        for (int jj = 0; jj < JT; ++jj)
#pragma unroll
          for (int e = 0; e < EPL; ++e) acc[jj][tt] = fmaf(wf[jj][e], xf[e], acc[jj][tt]);
      }
    }
  }
  __shared__ float red[4][JT][NB];
  const int wave = tid >> 6, lane = tid & 63;
#pragma unroll
  for (int jj = 0; jj < JT; ++jj)
#pragma unroll
    for (int tt = 0; tt < NB; ++tt) {
      const float s = wave_sum(acc[jj][tt]);
      if (lane == 0) red[wave][jj][tt] = s;
    }
  __syncthreads();
  if (tid < JT * NB) {
    const int jj = tid / NB, tt = tid % NB;
    if (j0 + jj < G3 && t0 + tt < ntok) {
      gi[size_t(t0 + tt) * G3 + j0 + jj] = (red[0][jj][tt] + red[1][jj][tt]) + (red[2][jj][tt] + red[3][jj][tt]);
    }
  }
}

__device__ inline float sigmoidf_(float a) { return 1.0f / (1.0f + expf(-a)); }

struct CellArgs {
  const void *W_hh;            // [3d'][d'] storage type
  const float *b_ih, *b_hh;    // [3d']
  const float *pos_w, *pos_b, *W1, *b1, *out_w, *out_b;
  const float *gi;             // [B*nsteps][3d'], token (b, i) at row b*nsteps + i
  float *z;                    // [B][d']
  float *score;                // [B][N_max]
  const float *override_;      // [B][override_stride] or null
  int override_stride;
  int dp, nsteps, pos0, N_max;
  float pos_scale;
};

// One workgroup per sequence; loops over `nsteps` consecutive tokens starting at position pos0.
template <typename T>
__global__ __launch_bounds__(512) void ctrl_cell_kernel(const CellArgs a) {
  extern __shared__ float smem[];
  const int dp = a.dp;
  float *h = smem;            // [dp]   z_{i-1}, then z_i
  float *gh = h + dp;         // [3dp]  W_hh h
  float *t_in = gh + 3 * dp;  // [dp]   p_i + z_i
  float *hn = t_in + dp;      // [dp]   z_i before it replaces h
  float *red = hn + dp;       // [8]    per-wave partial sums of the output layer
  const int b = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int nwaves = blockDim.x >> 6;
  const T *W_hh = static_cast<const T *>(a.W_hh);

  for (int j = tid; j < dp; j += blockDim.x) h[j] = a.z[size_t(b) * dp + j];
  __syncthreads();

  for (int i = 0; i < a.nsteps; ++i) {
    const float *gi = a.gi + (size_t(b) * a.nsteps + i) * 3 * dp;
    // recurrent pre-activations: one wave per row, lanes along the row
    for (int row = wave; row < 3 * dp; row += nwaves) {
      float s = 0.f;
      for (int t = lane; t < dp; t += 64) s = fmaf(to_float(W_hh[size_t(row) * dp + t]), h[t], s);
      s = wave_sum(s);
      if (lane == 0) gh[row] = s + a.b_hh[row];
    }
    __syncthreads();
    const float delta = float(a.pos0 + i) * a.pos_scale;
    for (int j = tid; j < dp; j += blockDim.x) {
      const float r = sigmoidf_(gi[j] + a.b_ih[j] + gh[j]);
      const float u = sigmoidf_(gi[dp + j] + a.b_ih[dp + j] + gh[dp + j]);
      const float cand = tanhf(gi[2 * dp + j] + a.b_ih[2 * dp + j] + r * gh[2 * dp + j]);
      const float hnew = (1.0f - u) * cand + u * h[j];
      hn[j] = hnew;
      t_in[j] = fmaf(a.pos_w[j], delta, a.pos_b[j]) + hnew;
    }
    __syncthreads();
    for (int j = tid; j < dp; j += blockDim.x) h[j] = hn[j];
    // interaction layer: one wave per row; output layer folded in
    float part = 0.f;
    for (int row = wave; row < dp; row += nwaves) {
      float s = 0.f;
      for (int t = lane; t < dp; t += 64) s = fmaf(a.W1[size_t(row) * dp + t], t_in[t], s);
      s = wave_sum(s);
      part = fmaf(a.out_w[row], tanhf(s + a.b1[row]), part);
    }
    if (lane == 0) red[wave] = part;
    __syncthreads();
    if (tid == 0) {
      float s = 0.f;
      for (int wv = 0; wv < nwaves; ++wv) s += red[wv];
      float sig = sigmoidf_(s + a.out_b[0]);
      if (a.override_) sig = a.override_[size_t(b) * a.override_stride + i];
      a.score[size_t(b) * a.N_max + a.pos0 + i] = sig;
    }
    __syncthreads();
  }
  for (int j = tid; j < dp; j += blockDim.x) a.z[size_t(b) * dp + j] = h[j];
}

}  // namespace

hipError_t launch_ctrl_input(adore_ctx *ctx, const void *x, int ntok, int per_seq, int seq_rows) {
  const adore_config &c = ctx->cfg;
  const int G3 = 3 * c.ctrl_hidden;
  dim3 grid((G3 + JT - 1) / JT, (ntok + NB - 1) / NB);
  ScopedTimer t(ctx, ADORE_KERNEL_CTRL_INPUT);
  if (c.dtype == ADORE_BF16) {
    hipLaunchKernelGGL((ctrl_input_kernel<bf16_t>), grid, dim3(256), 0, ctx->stream,
                       static_cast<const bf16_t *>(ctx->w.gru_w_ih), static_cast<const bf16_t *>(x), ctx->gi,
                       c.hidden, G3, ntok, per_seq, seq_rows);
  } else {
    hipLaunchKernelGGL((ctrl_input_kernel<float>), grid, dim3(256), 0, ctx->stream,
                       static_cast<const float *>(ctx->w.gru_w_ih), static_cast<const float *>(x), ctx->gi,
                       c.hidden, G3, ntok, per_seq, seq_rows);
  }
  return hipGetLastError();
}

hipError_t launch_ctrl_cell(adore_ctx *ctx, int nsteps, int pos0, const float *score_override,
                            int override_stride) {
  const adore_config &c = ctx->cfg;
  CellArgs a;
  a.W_hh = ctx->w.gru_w_hh;
  a.b_ih = ctx->w.gru_b_ih; a.b_hh = ctx->w.gru_b_hh;
  a.pos_w = ctx->w.pos_w; a.pos_b = ctx->w.pos_b;
  a.W1 = ctx->w.mlp_w1; a.b1 = ctx->w.mlp_b1;
  a.out_w = ctx->w.out_w; a.out_b = ctx->w.out_b;
  a.gi = ctx->gi; a.z = ctx->z; a.score = ctx->score;
  a.override_ = score_override; a.override_stride = override_stride;
  a.dp = c.ctrl_hidden; a.nsteps = nsteps; a.pos0 = pos0; a.N_max = c.max_positions;
  a.pos_scale = c.pos_scale;
  const size_t smem = size_t(6 * c.ctrl_hidden + 8) * sizeof(float);
  ScopedTimer t(ctx, ADORE_KERNEL_CTRL_CELL);
  if (c.dtype == ADORE_BF16) {
    hipLaunchKernelGGL((ctrl_cell_kernel<bf16_t>), dim3(c.batch), dim3(512), smem, ctx->stream, a);
  } else {
    hipLaunchKernelGGL((ctrl_cell_kernel<float>), dim3(c.batch), dim3(512), smem, ctx->stream, a);
  }
  return hipGetLastError();
}

}  // namespace adore
