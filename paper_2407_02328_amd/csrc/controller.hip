// Stage 2: the controller module (paper Sec. 2.2, Eq. 2; App. "Implementation
// Details": GRU input size D -> d', position layer 1 -> d', interaction layer
// d' -> d' with tanh, output layer d' -> 1 with sigmoid).
//
//   z_i     = GRU(x_i, z_{i-1})
//   sigma_i = sigmoid(out_w . tanh(W_1 (p_i + z_i) + b_1) + out_b),  p_i = pos_w * (i * pos_scale) + pos_b
//
// Two kernels.  ctrl_input computes the input pre-activations W_ih x for a
// batch of tokens: the only part that reads D-wide data, and free of any
// dependence between tokens, so a whole prompt chunk goes in one launch.  In
// bf16 it is a [tokens x D] x [D x 3d'] contraction on the matrix cores
// (16x16x32 tiles: 16 tokens x 16 gate rows), cut along D into `ksplit` slices
// so that a decode step (16 tokens) still spreads over many compute units; the
// slices are added up in a fixed order by the cell kernel.  ctrl_cell does the
// recurrent part token by token: W_hh z, the gates, the MLP and the score.
// All sums are fp32 in a fixed order, so results are reproducible run to run.
#include "device_utils.h"

namespace adore {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// ---- input projection, bf16, matrix cores -----------------------------------------
// grid (3d'/16, ceil(ntok/16), ksplit), 256 threads.  The workgroup owns a 16-token x 16-row
// tile and the D-slice z; its 4 waves cut the slice again and are summed through LDS.
// Inside a wave, lane group g = lane/16 walks the g-th quarter of the wave's k-range in
// 16-byte steps (both operands use the same assignment, so the order of k does not matter).
// part[z][tok][j] = sum over the slice of W_ih[j][k] * x_tok[k].
__global__ __launch_bounds__(256) void ctrl_input_mfma_kernel(const bf16_t *__restrict__ W_ih,
                                                              const bf16_t *__restrict__ x,
                                                              float *__restrict__ part, int D, int G3, int ntok,
                                                              int per_seq, int seq_rows, int kslice) {
  __builtin_amdgcn_s_setprio(3);   // short, latency-bound work that shares compute units with the GEMM: its waves go first
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int j0 = blockIdx.x * 16, t0 = blockIdx.y * 16;
  const int kw = kslice / 4;                       // k-range of one wave, a multiple of 32
  const int kbeg = blockIdx.z * kslice + wave * kw + (lane >> 4) * (kw / 4);
  int tok = t0 + (lane & 15);
  if (tok >= ntok) tok = ntok - 1;                 // padded rows read a valid token; dropped at the store
  const size_t xrow = size_t(tok / per_seq) * seq_rows + tok % per_seq;
  int j = j0 + (lane & 15);
  if (j >= G3) j = G3 - 1;
  const u32x4 *pa = reinterpret_cast<const u32x4 *>(x + xrow * D + kbeg);
  const u32x4 *pb = reinterpret_cast<const u32x4 *>(W_ih + size_t(j) * D + kbeg);
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  const int steps = kw / 32;                       // each MFMA consumes 32 k: 8 per lane group
  for (int s = 0; s < steps; ++s) {
    const u32x4 va = pa[s], vb = pb[s];
    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*reinterpret_cast<const bf16x8 *>(&va),
                                                  *reinterpret_cast<const bf16x8 *>(&vb), acc, 0, 0, 0);
  }
  // accumulator element v of lane L: token 4*(L/16) + v, gate row L%16
  __shared__ float red[4][16][17];
#pragma unroll
  for (int v = 0; v < 4; ++v) red[wave][4 * (lane >> 4) + v][lane & 15] = acc[v];
  __syncthreads();
  {
    const int m = tid >> 4, nn = tid & 15;
    if (t0 + m < ntok && j0 + nn < G3) {
      const float s = (red[0][m][nn] + red[1][m][nn]) + (red[2][m][nn] + red[3][m][nn]);
      part[(size_t(blockIdx.z) * ntok + t0 + m) * G3 + j0 + nn] = s;
    }
  }
}

// ---- input projection of a prompt chunk, bf16, matrix cores ---------------------------
// Thousands of tokens at once: a workgroup owns 64 tokens x 64 gate rows (4 x 4 tiles of the shape above)
// and the whole of D; its 4 waves cut D and keep all 16 tiles each, so a wave multiplies 16 tiles with
// 4 + 4 operand loads per step (the 16-token tile above re-reads W_ih once per 16 tokens and x once per
// 16 gate rows: at 8192 tokens that was 800 us).  The waves' sums are added in a fixed order.
// grid (ceil(3d'/64), ceil(ntok/64)), 256 threads.  gi[tok][j] (one D-slice).
__global__ __launch_bounds__(256) void ctrl_input_prompt_kernel(const bf16_t *__restrict__ W_ih,
                                                                const bf16_t *__restrict__ x,
                                                                float *__restrict__ gi, int D, int G3, int ntok,
                                                                int per_seq, int seq_rows) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int j0 = blockIdx.x * 64, t0 = blockIdx.y * 64;
  const int kw = D / 4;                            // k-range of one wave, a multiple of 32
  // a step of 32 k is one contiguous 64-byte run of every row, lane group g = lane/16 taking its g-th quarter
  // (with thousands of rows in flight, rows walked in four places at once would not stay in the L1)
  const int kbeg = wave * kw + (lane >> 4) * 8;
  const u32x4 *pa[4], *pb[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    int tok = t0 + 16 * i + (lane & 15);
    if (tok >= ntok) tok = ntok - 1;               // padded rows read a valid token; dropped at the store
    const size_t xrow = size_t(tok / per_seq) * seq_rows + tok % per_seq;
    pa[i] = reinterpret_cast<const u32x4 *>(x + xrow * D + kbeg);
    int j = j0 + 16 * i + (lane & 15);
    if (j >= G3) j = G3 - 1;
    pb[i] = reinterpret_cast<const u32x4 *>(W_ih + size_t(j) * D + kbeg);
  }
  f32x4 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) acc[i][jj] = f32x4{0.f, 0.f, 0.f, 0.f};
  const int steps = kw / 32;
#define PROMPT_STEP(VA, VB)                                                                                   \
  _Pragma("unroll") for (int i = 0; i < 4; ++i)                                                               \
    _Pragma("unroll") for (int jj = 0; jj < 4; ++jj)                                                          \
      acc[i][jj] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*reinterpret_cast<const bf16x8 *>(&VA[i]),         \
                                                           *reinterpret_cast<const bf16x8 *>(&VB[jj]), acc[i][jj], 0, 0, 0);
  int s = 0;
  for (; s + 2 <= steps; s += 2) {          // two steps' loads in flight
    u32x4 va[2][4], vb[2][4];
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int i = 0; i < 4; ++i) { va[u][i] = pa[i][(s + u) * 4]; vb[u][i] = pb[i][(s + u) * 4]; }
    PROMPT_STEP(va[0], vb[0])
    PROMPT_STEP(va[1], vb[1])
  }
  for (; s < steps; ++s) {
    u32x4 va[4], vb[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) { va[i] = pa[i][s * 4]; vb[i] = pb[i][s * 4]; }
    PROMPT_STEP(va, vb)
  }
#undef PROMPT_STEP
  // waves 3, 2, 1 hand their tiles to wave 0 through LDS, one after the other
  __shared__ float red[16][4][64];   // [tile][v][lane]: conflict-free, lane-private
  for (int w = 3; w >= 1; --w) {
    if (wave == w) {
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int jj = 0; jj < 4; ++jj)
#pragma unroll
          for (int v = 0; v < 4; ++v) red[i * 4 + jj][v][lane] = acc[i][jj][v];
    }
    __syncthreads();
    if (wave == 0) {
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int jj = 0; jj < 4; ++jj)
#pragma unroll
          for (int v = 0; v < 4; ++v) acc[i][jj][v] += red[i * 4 + jj][v][lane];
    }
    __syncthreads();
  }
  if (wave == 0) {   // accumulator element v of lane L: token 4*(L/16) + v, gate row L%16 of its tile
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int jj = 0; jj < 4; ++jj)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const int tok = t0 + 16 * i + 4 * (lane >> 4) + v, j = j0 + 16 * jj + (lane & 15);
          if (tok < ntok && j < G3) gi[size_t(tok) * G3 + j] = acc[i][jj][v];
        }
  }
}

// ---- input projection, any storage type, plain ALUs ---------------------------------
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
  const float *gi;             // [ksplit][B*nsteps][3d'], token (b, i) at row b*nsteps + i
  float *z;                    // [B][d']
  float *score;                // [B][N_max]
  float *cvec;                 // rescore mode: [B][N_max][d'] interaction-layer pre-activation at distance 0; else null
  const float *override_;      // [B][override_stride] or null
  int override_stride;
  int dp, nsteps, pos0, N_max, ksplit, ntok;
  float pos_scale;
};

// sum of the D-slices of one input pre-activation, in slice order; loads go out eight at a time
__device__ inline float gi_sum(const CellArgs &a, size_t tok, int j) {
  const size_t stride = size_t(a.ntok) * 3 * a.dp;
  const float *p = a.gi + tok * 3 * a.dp + j;
  float s = 0.f;
  int k = 0;
  for (; k + 16 <= a.ksplit; k += 16) {   // (sixteen at a time where there are that many: one trip to memory, same order)
    float v[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) v[u] = p[size_t(k + u) * stride];
#pragma unroll
    for (int u = 0; u < 16; ++u) s += v[u];
  }
  for (; k + 8 <= a.ksplit; k += 8) {
    float v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = p[size_t(k + u) * stride];
#pragma unroll
    for (int u = 0; u < 8; ++u) s += v[u];
  }
  for (; k < a.ksplit; ++k) s += p[size_t(k) * stride];
  return s;
}

// ---- cell, d' = 128 --------------------------------------------------------------------
// One workgroup of 4 waves per sequence, small enough in registers to share a compute unit with
// the rebuild GEMM of the previous step.  A weight row of 128 elements is one coalesced wave load
// (two elements per lane); a wave multiplies a batch of rows by the state it holds in registers and
// reduces the whole batch at once: at every halving step a lane keeps one half of its partial sums
// and hands the other half to its partner, so N rows cost N-1 shuffles instead of 6N.

// v[i] is this lane's partial sum of row i.  Returns, in every lane, the complete sum of row
// lane / (64 / N).
template <int N, int OFF>
struct ReduceRows {
  __device__ static inline float run(float (&v)[N], int lane) {
    const bool upper = (lane & OFF) != 0;
    float w[N / 2];
#pragma unroll
    for (int i = 0; i < N / 2; ++i) {
      const float keep = upper ? v[i + N / 2] : v[i];
      const float send = upper ? v[i] : v[i + N / 2];
      w[i] = keep + __shfl_xor(send, OFF, 64);
    }
    return ReduceRows<N / 2, OFF / 2>::run(w, lane);
  }
};
template <int OFF>
struct ReduceRows<1, OFF> {
  __device__ static inline float run(float (&v)[1], int) {
    float s = v[0];
#pragma unroll
    for (int off = OFF; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
    return s;
  }
};
template <int N>
__device__ inline float reduce_rows(float (&v)[N], int lane) {
  return ReduceRows<N, 32>::run(v, lane);
}

// two consecutive elements of a weight row, raw, and their conversion
__device__ inline uint32_t load_raw2(const bf16_t *p) { return *reinterpret_cast<const uint32_t *>(p); }
__device__ inline float2 load_raw2(const float *p) { return *reinterpret_cast<const float2 *>(p); }
__device__ inline float dot2(uint32_t u, float x0, float x1) {
  return fmaf(__uint_as_float(u << 16), x0, __uint_as_float(u & 0xffff0000u) * x1);
}
__device__ inline float dot2(float2 u, float x0, float x1) { return fmaf(u.x, x0, u.y * x1); }

// out[row0 + r] = bias[row0 + r] + W[row0 + r][:] . x   for r < N, x held as (x0, x1) = x[2*lane], x[2*lane+1]
template <typename T, int N>
__device__ inline void rows_times_vec(const T *W, int row0, float x0, float x1, const float *bias, float *out,
                                      int lane) {
  decltype(load_raw2(W)) raw[N];
#pragma unroll
  for (int i = 0; i < N; ++i) raw[i] = load_raw2(W + size_t(row0 + i) * 128 + 2 * lane);
  __builtin_amdgcn_sched_barrier(0);   // all N loads go out before the first is waited for
  float v[N];
#pragma unroll
  for (int i = 0; i < N; ++i) v[i] = dot2(raw[i], x0, x1);
  const float s = reduce_rows<N>(v, lane);
  constexpr int LPRW = 64 / N;   // lanes holding the same row
  if ((lane & (LPRW - 1)) == 0) {
    const int r = row0 + lane / LPRW;
    out[r] = s + bias[r];
  }
}

// The same product in two halves: the N row loads go out where the caller wants them (next to everything else a
// step reads), the arithmetic follows once x is known.
template <typename T, int N>
__device__ inline void rows_request(const T *W, int row0, int lane, decltype(load_raw2(W)) (&raw)[N]) {
#pragma unroll
  for (int i = 0; i < N; ++i) raw[i] = load_raw2(W + size_t(row0 + i) * 128 + 2 * lane);
}
template <typename R, int N>
__device__ inline void rows_finish(const R (&raw)[N], int row0, float x0, float x1, const float *bias, float *out, int lane) {
  float v[N];
#pragma unroll
  for (int i = 0; i < N; ++i) v[i] = dot2(raw[i], x0, x1);
  const float s = reduce_rows<N>(v, lane);
  constexpr int LPRW = 64 / N;   // lanes holding the same row
  if ((lane & (LPRW - 1)) == 0) {
    const int r = row0 + lane / LPRW;
    out[r] = s + bias[r];
  }
}

// One token per sequence (a decode step).  One workgroup of 12 waves per sequence.  A step's cost is not its
// arithmetic (100 k multiply-adds) but its trips to memory, each of which takes microseconds next to the
// attention's traffic: so everything the step reads is requested at the top, before anything is waited for: the
// state, the D-slices of the input pre-activations, W_hh (32 rows per wave), W_1 (32 rows each for 4 of the
// waves), the small vectors.  After that the kernel only computes, with three barriers.
template <typename T>
__global__ __launch_bounds__(768) void ctrl_cell128_kernel(const CellArgs a) {
  __builtin_amdgcn_s_setprio(3);   // short, latency-bound work next to the attention: its waves go first
  constexpr int DP = 128;
  __shared__ float gi_s[3 * DP];   // W_ih x + b_ih
  __shared__ float gh[3 * DP];     // W_hh h + b_hh
  __shared__ float t_in[DP];       // p_i + z_i
  __shared__ float u1[DP];         // W_1 (p + z) + b_1
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const T *W_hh = static_cast<const T *>(a.W_hh);
  const size_t tok = size_t(b);    // nsteps == 1
  // ---- requests ----
  const float2 hx = *reinterpret_cast<const float2 *>(a.z + size_t(b) * DP + 2 * lane);   // z_{i-1}, in every wave
  decltype(load_raw2(W_hh)) rhh[32];
  rows_request<T, 32>(W_hh, wave * 32, lane, rhh);
  float2 rw1[32];                  // (batches of 32 rows, as where a prompt chunk is scored: the same sums in the same order)
  if (wave < 4) rows_request<float, 32>(a.W1, wave * 32, lane, rw1);
  float g = 0.f, hold = 0.f, pw = 0.f, pb = 0.f, ow0 = 0.f, ow1 = 0.f, ob = 0.f, ov = 0.f;
  if (tid < 3 * DP) g = gi_sum(a, tok, tid) + a.b_ih[tid];
  if (tid < DP) {
    hold = a.z[size_t(b) * DP + tid];
    pw = a.pos_w[tid];
    pb = a.pos_b[tid];
  }
  if (wave == 0) {
    ow0 = a.out_w[lane];
    ow1 = a.out_w[lane + 64];
    ob = a.out_b[0];
    if (a.override_) ov = a.override_[size_t(b) * a.override_stride];
  }
  __builtin_amdgcn_sched_barrier(0);   // all of the above is under way before the first use
  // ---- recurrent pre-activations, the gates, the new state ----
  rows_finish<decltype(load_raw2(W_hh)), 32>(rhh, wave * 32, hx.x, hx.y, a.b_hh, gh, lane);
  if (tid < 3 * DP) gi_s[tid] = g;
  __syncthreads();
  if (tid < DP) {
    const float r = sigmoidf_(gi_s[tid] + gh[tid]);
    const float u = sigmoidf_(gi_s[DP + tid] + gh[DP + tid]);
    const float cand = tanhf(gi_s[2 * DP + tid] + r * gh[2 * DP + tid]);
    const float hnew = (1.0f - u) * cand + u * hold;
    const float delta = a.cvec ? 0.f : float(a.pos0) * a.pos_scale;   // rescore mode: distance to itself
    a.z[size_t(b) * DP + tid] = hnew;
    t_in[tid] = fmaf(pw, delta, pb) + hnew;
  }
  __syncthreads();
  // ---- interaction layer, output layer, sigmoid ----
  if (wave < 4) rows_finish<float2, 32>(rw1, wave * 32, t_in[2 * lane], t_in[2 * lane + 1], a.b1, u1, lane);
  __syncthreads();
  if (a.cvec && tid < DP) a.cvec[(size_t(b) * a.N_max + a.pos0) * DP + tid] = u1[tid];
  if (wave == 0) {
    float s = fmaf(ow0, tanhf(u1[lane]), ow1 * tanhf(u1[lane + 64]));
    s = wave_sum(s);
    if (lane == 0) a.score[size_t(b) * a.N_max + a.pos0] = a.override_ ? ov : sigmoidf_(s + ob);
  }
}

// ---- a prompt chunk, d' = 128: the recurrence alone, then the layers above it for all tokens at once ----
// Only z_i = GRU(x_i, z_{i-1}) ties a token to the one before it; the position, interaction and output layers
// do not.  The scan therefore does nothing but the recurrence, one workgroup of 4 waves per sequence, with W_hh
// in registers as fp32 for the whole chunk: wave w keeps columns 32w .. 32w+31 of all 384 rows (lane l: rows
// l, l+64, .., l+320), so a token costs a wave 8 16-byte reads of the state from LDS (same address in every
// lane) and 192 multiply-adds per lane on each of the four SIMDs; the four partial sums of a row meet in LDS,
// 128 threads apply the gates.  Two barriers and no memory round trip per token.  The gates use the hardware's exp2 and reciprocal
// (about 2e-7 absolute); z_i goes to zseq[b * nsteps + i][128] for the kernel below.
__device__ inline float scan_sigmoid(float a) {
  return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.44269504f * a));
}
__device__ inline float scan_tanh(float a) {
  return 1.0f - 2.0f * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(2.88539008f * a));
}

template <typename T>
__global__ __launch_bounds__(256) void ctrl_scan128_kernel(const CellArgs a, float *__restrict__ zseq) {
  constexpr int DP = 128, KW = 32, RPL = 6;               // columns per wave, rows per lane
  constexpr int TB = 16, GPT = TB * (3 * DP / 4) / 256;   // tokens per block of input pre-activations; float4 per thread
  __shared__ __attribute__((aligned(16))) float h[DP];   // z_{i-1}, then z_i
  __shared__ float part[4][3 * DP];                        // the waves' partial sums of W_hh h
  __shared__ float4 gbuf[2][TB * (3 * DP / 4)];            // input pre-activations of two blocks of tokens
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  float w[RPL][KW];
  {
    constexpr int EPL = Vec16<T>::EPL;
#pragma unroll
    for (int m = 0; m < RPL; ++m) {
      const T *row = static_cast<const T *>(a.W_hh) + size_t(lane + 64 * m) * DP + wave * KW;
#pragma unroll
      for (int c = 0; c < KW; c += EPL) {
        float f[EPL];
        Vec16<T>::load(row + c, f);
#pragma unroll
        for (int e = 0; e < EPL; ++e) w[m][c + e] = f[e];
      }
    }
  }
  float b_r = 0.f, b_u = 0.f, b_in = 0.f, b_hn = 0.f, hcur = 0.f;
  if (tid < DP) {
    hcur = a.z[size_t(b) * DP + tid];
    h[tid] = hcur;
    b_r = a.b_ih[tid] + a.b_hh[tid];
    b_u = a.b_ih[DP + tid] + a.b_hh[DP + tid];
    b_in = a.b_ih[2 * DP + tid];
    b_hn = a.b_hh[2 * DP + tid];
  }
  // The input pre-activations reach the gates through LDS, TB tokens at a time: the rows of block j+1 are
  // fetched (all threads, 16 bytes each, the D-slices added up) while block j is worked through, so the
  // recurrence never waits for memory.
  const int nblk = (a.nsteps + TB - 1) / TB;
  const float4 *gsrc = reinterpret_cast<const float4 *>(a.gi) + size_t(b) * a.nsteps * (3 * DP / 4);
  const size_t slice4 = size_t(a.ntok) * (3 * DP / 4);   // distance between two D-slices
  float4 stage[GPT];
  auto fetch = [&](int blk) {
    const int rows = a.nsteps - blk * TB < TB ? a.nsteps - blk * TB : TB;
#pragma unroll
    for (int q = 0; q < GPT; ++q) {
      const int idx = tid + 256 * q;
      float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
      if (idx < rows * (3 * DP / 4)) {
        const float4 *p = gsrc + size_t(blk) * TB * (3 * DP / 4) + idx;
        v = p[0];
        for (int k = 1; k < a.ksplit; ++k) {
          const float4 t = p[size_t(k) * slice4];
          v.x += t.x; v.y += t.y; v.z += t.z; v.w += t.w;
        }
      }
      stage[q] = v;
    }
  };
  auto park = [&](int buf) {
#pragma unroll
    for (int q = 0; q < GPT; ++q) gbuf[buf][tid + 256 * q] = stage[q];
  };
  if (nblk > 0) {
    fetch(0);
    park(0);
  }
  __syncthreads();
  for (int blk = 0; blk < nblk; ++blk) {
    if (blk + 1 < nblk) fetch(blk + 1);
    const float *g = reinterpret_cast<const float *>(gbuf[blk & 1]);
    const int rows = a.nsteps - blk * TB < TB ? a.nsteps - blk * TB : TB;
    for (int ii = 0; ii < rows; ++ii) {
      const size_t tok = size_t(b) * a.nsteps + blk * TB + ii;
      float acc[RPL];
#pragma unroll
      for (int m = 0; m < RPL; ++m) acc[m] = 0.f;
#pragma unroll
      for (int k = 0; k < KW; k += 4) {
        const float4 hv = *reinterpret_cast<const float4 *>(&h[wave * KW + k]);
#pragma unroll
        for (int m = 0; m < RPL; ++m) {
          acc[m] = fmaf(w[m][k], hv.x, acc[m]);
          acc[m] = fmaf(w[m][k + 1], hv.y, acc[m]);
          acc[m] = fmaf(w[m][k + 2], hv.z, acc[m]);
          acc[m] = fmaf(w[m][k + 3], hv.w, acc[m]);
        }
      }
#pragma unroll
      for (int m = 0; m < RPL; ++m) part[wave][lane + 64 * m] = acc[m];
      __syncthreads();
      if (tid < DP) {
        const float s_r = (part[0][tid] + part[1][tid]) + (part[2][tid] + part[3][tid]);
        const float s_u = (part[0][DP + tid] + part[1][DP + tid]) + (part[2][DP + tid] + part[3][DP + tid]);
        const float s_n = (part[0][2 * DP + tid] + part[1][2 * DP + tid]) + (part[2][2 * DP + tid] + part[3][2 * DP + tid]);
        const float *gt = g + ii * 3 * DP;
        const float r = scan_sigmoid(gt[tid] + b_r + s_r);
        const float u = scan_sigmoid(gt[DP + tid] + b_u + s_u);
        const float cand = scan_tanh(gt[2 * DP + tid] + b_in + r * (s_n + b_hn));
        hcur = (1.0f - u) * cand + u * hcur;
        h[tid] = hcur;
        zseq[tok * DP + tid] = hcur;
      }
      __syncthreads();
    }
    if (blk + 1 < nblk) park((blk + 1) & 1);   // read next after at least one more barrier
  }
  if (tid < DP) a.z[size_t(b) * DP + tid] = hcur;
}

// sigma_i = sigmoid(out_w . tanh(W_1 (p_i + z_i) + b_1) + out_b) for the tokens of a chunk, from the z_i the scan
// left.  grid (ceil(nsteps / 16), B), 4 waves, 4 tokens per wave one after the other; the arithmetic is the cell
// kernel's (rows_times_vec, same order), so a token scored here and one scored by a step agree bit for bit
// given the same z_i.
__global__ __launch_bounds__(256) void ctrl_mlp128_kernel(const CellArgs a, const float *__restrict__ zseq) {
  constexpr int DP = 128;
  __shared__ float u1[4][DP];
  const int b = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  for (int q = 0; q < 4; ++q) {
    const int i = blockIdx.x * 16 + wave * 4 + q;
    const bool on = i < a.nsteps;                      // uniform over the wave; the barriers are not skipped
    const size_t tok = size_t(b) * a.nsteps + (on ? i : 0);
    const float delta = a.cvec ? 0.f : float(a.pos0 + i) * a.pos_scale;   // rescore mode: distance to itself
    const float x0 = fmaf(a.pos_w[2 * lane], delta, a.pos_b[2 * lane]) + zseq[tok * DP + 2 * lane];
    const float x1 = fmaf(a.pos_w[2 * lane + 1], delta, a.pos_b[2 * lane + 1]) + zseq[tok * DP + 2 * lane + 1];
#pragma unroll 1
    for (int part = 0; part < 4; ++part) rows_times_vec<float, 32>(a.W1, part * 32, x0, x1, a.b1, u1[wave], lane);
    __syncthreads();
    if (on) {
      if (a.cvec) {
        float *c = a.cvec + (size_t(b) * a.N_max + a.pos0 + i) * DP;
        c[lane] = u1[wave][lane];
        c[lane + 64] = u1[wave][lane + 64];
      }
      float s = fmaf(a.out_w[lane], tanhf(u1[wave][lane]), a.out_w[lane + 64] * tanhf(u1[wave][lane + 64]));
      s = wave_sum(s);
      if (lane == 0) {
        float sig = sigmoidf_(s + a.out_b[0]);
        if (a.override_) sig = a.override_[size_t(b) * a.override_stride + i];
        a.score[size_t(b) * a.N_max + a.pos0 + i] = sig;
      }
    }
    __syncthreads();
  }
}

// ---- cell, any d' -------------------------------------------------------------------
// One workgroup per sequence; loops over `nsteps` consecutive tokens starting at position pos0.
template <typename T>
__global__ __launch_bounds__(512) void ctrl_cell_kernel(const CellArgs a) {
  __builtin_amdgcn_s_setprio(3);   // short, latency-bound work that shares compute units with the GEMM: its waves go first
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
    const size_t tok = size_t(b) * a.nsteps + i;
    // recurrent pre-activations: one wave per row, lanes along the row
    for (int row = wave; row < 3 * dp; row += nwaves) {
      float s = 0.f;
      for (int t = lane; t < dp; t += 64) s = fmaf(to_float(W_hh[size_t(row) * dp + t]), h[t], s);
      s = wave_sum(s);
      if (lane == 0) gh[row] = s + a.b_hh[row];
    }
    __syncthreads();
    const float delta = a.cvec ? 0.f : float(a.pos0 + i) * a.pos_scale;   // rescore mode: distance to itself
    for (int j = tid; j < dp; j += blockDim.x) {
      const float r = sigmoidf_(gi_sum(a, tok, j) + a.b_ih[j] + gh[j]);
      const float u = sigmoidf_(gi_sum(a, tok, dp + j) + a.b_ih[dp + j] + gh[dp + j]);
      const float cand = tanhf(gi_sum(a, tok, 2 * dp + j) + a.b_ih[2 * dp + j] + r * gh[2 * dp + j]);
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
      if (a.cvec && lane == 0) a.cvec[(size_t(b) * a.N_max + a.pos0 + i) * dp + row] = s + a.b1[row];
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

// ---- rescore mode -----------------------------------------------------------------
// W_1 (pos_w * delta + pos_b + z_i) + b_1  =  c_i + delta * a   with  c_i = W_1 (z_i + pos_b) + b_1  kept per
// token by the cell kernels and  a = W_1 pos_w:  scoring a token again costs d' tanh and one dot product.
__global__ __launch_bounds__(256) void ctrl_avec_kernel(const float *__restrict__ W1,
                                                        const float *__restrict__ pos_w,
                                                        float *__restrict__ avec, int dp) {
  for (int row = threadIdx.x; row < dp; row += blockDim.x) {
    float s = 0.f;
    for (int k = 0; k < dp; ++k) s = fmaf(W1[size_t(row) * dp + k], pos_w[k], s);
    avec[row] = s;
  }
}

// sigma_i(n) = sigmoid(out_w . tanh(c_i + (n - i) * pos_scale * a) + out_b) for i = 0..upto.  16 lanes per
// token, 16 tokens per workgroup; grid = (tokens / 16, B).  In a step upto = n - 1: the current token's score (distance
// 0) is the cell kernel's, which runs next to this one.
__global__ __launch_bounds__(256) void rescore_kernel(const float *__restrict__ cvec,
                                                      const float *__restrict__ avec,
                                                      const float *__restrict__ out_w,
                                                      const float *__restrict__ out_b,
                                                      float *__restrict__ score, int n, int upto, int N_max,
                                                      int dp, float pos_scale) {
  __builtin_amdgcn_s_setprio(3);   // short, latency-bound work that shares compute units with the GEMM: its waves go first
  const int b = blockIdx.y;
  const int i = blockIdx.x * 16 + (threadIdx.x >> 4);
  const int lig = threadIdx.x & 15;
  const int ic = i <= upto ? i : upto;           // lanes past the end redo the last token and store nothing
  const float delta = float(n - ic) * pos_scale;
  const float *c = cvec + (size_t(b) * N_max + ic) * dp;
  float s = 0.f;
  for (int e = lig * 4; e < dp; e += 64) {
    const float4 cv = *reinterpret_cast<const float4 *>(c + e);
    const float4 av = *reinterpret_cast<const float4 *>(avec + e);
    const float4 wv = *reinterpret_cast<const float4 *>(out_w + e);
    s = fmaf(wv.x, tanhf(fmaf(delta, av.x, cv.x)), s);
    s = fmaf(wv.y, tanhf(fmaf(delta, av.y, cv.y)), s);
    s = fmaf(wv.z, tanhf(fmaf(delta, av.z, cv.z)), s);
    s = fmaf(wv.w, tanhf(fmaf(delta, av.w, cv.w)), s);
  }
#pragma unroll
  for (int off = 8; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
  if (lig == 0 && i <= upto) score[size_t(b) * N_max + i] = sigmoidf_(s + out_b[0]);
}

// Number of D-slices of the bf16 input projection: enough workgroups to cover the chip when
// there are few tokens, and slices short enough that a wave walks at most four 32-wide steps of its quarter (the
// operand loads of a step touch 64 cache lines and wait for each other: at 128 tokens, two slices of 2048 took
// 225 us); one slice when there are many tokens.  A slice is a multiple of 128 (4 waves x 32).
int ctrl_input_ksplit(const adore_config &c, int ntok) {
  const int tiles = ((3 * c.ctrl_hidden + 15) / 16) * ((ntok + 15) / 16);
  int ks = 1;
  if (ntok > kCtrlSplitTokens) return 1;
  while (ks < kMaxCtrlSplit && (tiles * ks < 256 || c.hidden / ks > 512) && c.hidden % (ks * 2 * 128) == 0) ks *= 2;
  return ks;
}

}  // namespace

hipError_t launch_ctrl_input(adore_ctx *ctx, hipStream_t st, const void *x, int ntok, int per_seq,
                             int seq_rows, int *ksplit_out) {
  const adore_config &c = ctx->cfg;
  const int G3 = 3 * c.ctrl_hidden;
  ScopedTimer t(ctx, ADORE_KERNEL_CTRL_INPUT, st);
  *ksplit_out = 1;
  if (ntok > kCtrlSplitTokens &&
      launch_plain_projection(ctx, t, st, x, ctx->w.gru_w_ih, ctx->gi, ntok, per_seq, seq_rows, G3, c.hidden)) {
    // a prompt chunk on the rebuild's 128x128 tile (3d' a multiple of 128, D of 64)
  } else if (c.dtype == ADORE_BF16 && c.hidden % 128 == 0 && ntok > kCtrlSplitTokens) {
    dim3 grid((G3 + 63) / 64, (ntok + 63) / 64);
    ADORE_LAUNCH(t, ctrl_input_prompt_kernel, grid, dim3(256), 0, st,
                       static_cast<const bf16_t *>(ctx->w.gru_w_ih), static_cast<const bf16_t *>(x), ctx->gi,
                       c.hidden, G3, ntok, per_seq, seq_rows);
  } else if (c.dtype == ADORE_BF16 && c.hidden % 128 == 0) {
    const int ks = ctrl_input_ksplit(c, ntok);
    *ksplit_out = ks;
    dim3 grid((G3 + 15) / 16, (ntok + 15) / 16, ks);
    ADORE_LAUNCH(t, ctrl_input_mfma_kernel, grid, dim3(256), 0, st,
                       static_cast<const bf16_t *>(ctx->w.gru_w_ih), static_cast<const bf16_t *>(x), ctx->gi,
                       c.hidden, G3, ntok, per_seq, seq_rows, c.hidden / ks);
  } else if (c.dtype == ADORE_BF16) {
    dim3 grid((G3 + JT - 1) / JT, (ntok + NB - 1) / NB);
    ADORE_LAUNCH(t, (ctrl_input_kernel<bf16_t>), grid, dim3(256), 0, st,
                       static_cast<const bf16_t *>(ctx->w.gru_w_ih), static_cast<const bf16_t *>(x), ctx->gi,
                       c.hidden, G3, ntok, per_seq, seq_rows);
  } else {
    dim3 grid((G3 + JT - 1) / JT, (ntok + NB - 1) / NB);
    ADORE_LAUNCH(t, (ctrl_input_kernel<float>), grid, dim3(256), 0, st,
                       static_cast<const float *>(ctx->w.gru_w_ih), static_cast<const float *>(x), ctx->gi,
                       c.hidden, G3, ntok, per_seq, seq_rows);
  }
  return hipGetLastError();
}

hipError_t launch_ctrl_cell(adore_ctx *ctx, hipStream_t st, int nsteps, int pos0,
                            const float *score_override, int override_stride, int ksplit) {
  const adore_config &c = ctx->cfg;
  CellArgs a;
  a.W_hh = ctx->w.gru_w_hh;
  a.b_ih = ctx->w.gru_b_ih; a.b_hh = ctx->w.gru_b_hh;
  a.pos_w = ctx->w.pos_w; a.pos_b = ctx->w.pos_b;
  a.W1 = ctx->w.mlp_w1; a.b1 = ctx->w.mlp_b1;
  a.out_w = ctx->w.out_w; a.out_b = ctx->w.out_b;
  a.gi = ctx->gi; a.z = ctx->z; a.score = ctx->score;
  a.cvec = c.score_mode == ADORE_SCORE_RESCORE ? ctx->cvec : nullptr;
  a.override_ = score_override; a.override_stride = override_stride;
  a.dp = c.ctrl_hidden; a.nsteps = nsteps; a.pos0 = pos0; a.N_max = c.max_positions;
  a.ksplit = ksplit; a.ntok = c.batch * nsteps;
  a.pos_scale = c.pos_scale;
  if (c.ctrl_hidden == 128 && nsteps > 1) {   // a prompt chunk: the recurrence, then the layers above it
    {
      ScopedTimer t(ctx, ADORE_KERNEL_CTRL_CELL, st);
      if (c.dtype == ADORE_BF16) {
        ADORE_LAUNCH(t, (ctrl_scan128_kernel<bf16_t>), dim3(c.batch), dim3(256), 0, st, a, ctx->zseq);
      } else {
        ADORE_LAUNCH(t, (ctrl_scan128_kernel<float>), dim3(c.batch), dim3(256), 0, st, a, ctx->zseq);
      }
    }
    ScopedTimer t(ctx, ADORE_KERNEL_CTRL_CELL, st);
    ADORE_LAUNCH(t, ctrl_mlp128_kernel, dim3((nsteps + 15) / 16, c.batch), dim3(256), 0, st, a,
                 static_cast<const float *>(ctx->zseq));
    return hipGetLastError();
  }
  ScopedTimer t(ctx, ADORE_KERNEL_CTRL_CELL, st);
  if (c.ctrl_hidden == 128) {
    if (c.dtype == ADORE_BF16) {
      ADORE_LAUNCH(t, (ctrl_cell128_kernel<bf16_t>), dim3(c.batch), dim3(768), 0, st, a);
    } else {
      ADORE_LAUNCH(t, (ctrl_cell128_kernel<float>), dim3(c.batch), dim3(768), 0, st, a);
    }
  } else {
    const size_t smem = size_t(6 * c.ctrl_hidden + 8) * sizeof(float);
    if (c.dtype == ADORE_BF16) {
      ADORE_LAUNCH(t, (ctrl_cell_kernel<bf16_t>), dim3(c.batch), dim3(512), smem, st, a);
    } else {
      ADORE_LAUNCH(t, (ctrl_cell_kernel<float>), dim3(c.batch), dim3(512), smem, st, a);
    }
  }
  return hipGetLastError();
}

hipError_t launch_ctrl_avec(adore_ctx *ctx, hipStream_t st) {
  hipLaunchKernelGGL(ctrl_avec_kernel, dim3(1), dim3(256), 0, st, ctx->w.mlp_w1, ctx->w.pos_w, ctx->avec,
                     ctx->cfg.ctrl_hidden);
  return hipGetLastError();
}

hipError_t launch_rescore(adore_ctx *ctx, hipStream_t st, int n, int upto) {
  const adore_config &c = ctx->cfg;
  if (upto < 0) return hipSuccess;
  ScopedTimer t(ctx, ADORE_KERNEL_RESCORE, st);
  ADORE_LAUNCH(t, rescore_kernel, dim3((upto + 16) / 16, c.batch), dim3(256), 0, st, ctx->cvec, ctx->avec,
               ctx->w.out_w, ctx->w.out_b, ctx->score, n, upto, c.max_positions, c.ctrl_hidden, c.pos_scale);
  return hipGetLastError();
}

}  // namespace adore
