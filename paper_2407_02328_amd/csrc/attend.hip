// Stage 1: insert the current token's k, v and single-query attention over the
// occupied slots of every (sequence, head)  (paper Sec. 2.1: Eq. 1 restricted to
// the retained rows plus the current token).
//
// Memory-bound: every step streams K*d*2 elements of K and V per row once.  A
// row of d elements is 16-byte vectors spread over LPR consecutive lanes, so a
// wave reads 64/LPR whole cache rows (1 KB, contiguous) per load instruction.
// The slots of one (b,h) are cut into `nsplit` chunks, one workgroup each, so
// that small batches still fill the chip; partial (max, sum, acc) triples are
// merged by a second small kernel (a merge inside the first kernel would need a
// device-scope release per workgroup, which on a multi-XCD part writes back the
// whole L2 and costs far more than the extra launch).  When there are enough
// rows, one workgroup of up to 16 waves takes a whole row and no merge kernel
// runs.  Softmax runs online in fp32, base 2.
#include <cstdlib>

#include "select_device.h"

namespace adore {

namespace {

// The step's two selections as extra workgroups of the attention launch (static score mode: neither selection
// of step n looks at the current token's score, so they depend on nothing this launch computes, and nothing in
// this launch depends on them).  Per sequence: rel_wgs workgroups release heads 1 .. H-1 (one wave per head),
// one more releases head 0 and then chooses the tokens to rebuild from the positions head 0 keeps.
// The chosen positions are entered into the slot maps by the kernel that writes their rows.
struct SchedArgs {
  int kpl, rel_wgs;                 // keys per lane of a row (K / 64 rounded up to 2, 4, 8, 16); 0 workgroups = off
  int prio;                         // wave priority of the role (0 .. 3)
  int hpw;                          // heads a wave releases one after the other (1, or 4 for short rows of many sequences)
  const int32_t *slot_src;          // [B*H][K]
  int32_t *slot_dst;                // [B*H][K]
  const float *score;               // [B][N_max]
  int32_t *free_list;               // [B*H][R1]
  int32_t *released_pos, *map_out, *rel_out;
  int H, K, N_max, n, x, R1;
  RebuildSelectArgs sel;
};

struct AttendArgs {
  const void *q, *k_new, *v_new;   // [B*H][d]
  void *Kc, *Vc;                   // [B*H][K][d] of this layer
  const int32_t *slot_pos;         // [B*H][K]
  const int32_t *insert_slot;      // the reserved slot of row bh is insert_slot[bh * ins_stride + ins_off]
  int ins_stride, ins_off;
  int n_sel;                       // the first n_sel workgroups carry the selections (they start first: their chain
                                   // of dependent steps is the longest), the attention's come behind them
  SchedArgs s;
  float *part;                     // [B*H][nsplit][d+2]
  float *out;                      // [B*H][d]
  float *logit_out;                // null, or [B*H][K]: every slot's logit as scaled here (base 2; -inf for a free slot)
  float *ml_out;                   // ... and [B*H][2]: the row's maximum logit and the sum of exp2(logit - maximum),
                                   // from which a row's probabilities follow (the scores of the H2O mode)
  int K, chunk, nsplit;
  float scale_log2;                // log2(e) / sqrt(d)
};

// Dynamic LDS of a workgroup in this role: [scores of the sequence, n + 1 floats][head 0's row, K ints][choice].
// The scores are copied once and the rows are read at the same time, so that afterwards the ranking keys come
// from LDS: under the attention's traffic every dependent trip to memory costs five to seven microseconds.
// hist: 256 words of LDS per wave for the release's radix select (the attention's own merge buffer, which these
// workgroups do not use otherwise).
template <int WAVES, int KPL>
__device__ inline void selections_role(const AttendArgs &a, int e, uint64_t *dyn, uint32_t *hist) {
  // Rows short enough to fit four of them into a wave's registers can be released four to a wave: with hundreds of
  // sequences the role's workgroups would otherwise take half of the chip's wave slots from the attention for the
  // time their trips to memory take.
  constexpr int HPW = KPL <= 4 ? 4 : 1;
  const SchedArgs &s = a.s;
  const int per_seq = s.rel_wgs + 1;
  const int b = e / per_seq, part = e - b * per_seq;
  const int tid = threadIdx.x, wave = tid >> 6;
  switch (s.prio) {   // few waves with a long chain of dependent steps
    case 3: __builtin_amdgcn_s_setprio(3); break;
    case 2: __builtin_amdgcn_s_setprio(2); break;
    case 1: __builtin_amdgcn_s_setprio(1); break;
    default: break;
  }
  float *s_score = reinterpret_cast<float *>(dyn);
  const float *sc = s.score + size_t(b) * s.N_max;
  if (part < s.rel_wgs) {          // heads 1 .. H-1
    const int hpw = HPW > 1 ? s.hpw : 1;
    const int h0 = 1 + (part * WAVES + wave) * hpw;
    int raw[HPW][KPL], s_ins[HPW];
#pragma unroll
    for (int i = 0; i < HPW; ++i) {
      if (i < hpw && h0 + i < s.H) {   // whole waves
        const int row = b * s.H + h0 + i;
        s_ins[i] = a.insert_slot[size_t(row) * a.ins_stride + a.ins_off];
        release_fetch<KPL>(row, s.slot_src, s.K, raw[i]);
      }
    }
    for (int i = tid; i <= s.n; i += 64 * WAVES) s_score[i] = sc[i];
    __syncthreads();
#pragma unroll
    for (int i = 0; i < HPW; ++i) {
      if (i < hpw && h0 + i < s.H)
        release_row<KPL>(b * s.H + h0 + i, s_ins[i], s.slot_src, s.slot_dst, s_score, s.free_list, s.released_pos, s.map_out,
                         s.rel_out, s.K, s.n, s.x, s.R1, nullptr, hist + wave * 256, raw[i]);
    }
    return;
  }
  // head 0, then the choice of the tokens to rebuild from the positions it keeps
  const int row = b * s.H;
  const int s_ins = a.insert_slot[size_t(row) * a.ins_stride + a.ins_off];
  int raw[KPL];
  if (wave == 0) release_fetch<KPL>(row, s.slot_src, s.K, raw);
  for (int i = tid; i <= s.n; i += 64 * WAVES) s_score[i] = sc[i];
  __syncthreads();
  int32_t *row_copy = reinterpret_cast<int32_t *>(dyn + (s.n + 2) / 2);   // head 0's positions after the release
  uint64_t *choice = dyn + (s.n + 2) / 2 + (s.K + 1) / 2;
  if (wave == 0) {
    release_row<KPL>(row, s_ins, s.slot_src, s.slot_dst, s_score, s.free_list, s.released_pos, s.map_out,
                     s.rel_out, s.K, s.n, s.x, s.R1, row_copy, hist, raw);
  } else {
    choice_fill_keys(s_score, s.n, choice, tid - 64, 64 * (WAVES - 1));   // the other waves meanwhile
  }
  __syncthreads();
  choice_from_keys(s.sel, b, row_copy, choice);
}

template <typename T, int DH, int U, int WAVES>
__global__ __launch_bounds__(64 * WAVES, 4) void attend_kernel(const AttendArgs a) {
  constexpr int EPL = Vec16<T>::EPL;    // elements per lane
  constexpr int LPR = DH / EPL;         // lanes per cache row
  constexpr int RPW = 64 / LPR;         // rows per wave and load
  constexpr int G = WAVES * RPW;        // lane groups (rows in flight) per workgroup
  static_assert(LPR >= 1 && LPR <= 64 && (LPR & (LPR - 1)) == 0, "row must be a power-of-two lane group");
  // merge of the lane groups at the end of a row; a workgroup that carries selections instead keeps its waves'
  // radix histograms there
  __shared__ float s_m[G], s_l[G];
  __shared__ float s_acc[G][DH];
  static_assert(G * DH >= WAVES * 256, "room for one 256-bin histogram per wave");

  if (int(blockIdx.x) < a.n_sel) {   // uniform over the workgroup
    extern __shared__ uint64_t dyn_smem[];
    const int e = blockIdx.x;
    uint32_t *hist = reinterpret_cast<uint32_t *>(&s_acc[0][0]);
    switch (a.s.kpl) {
      case 2: selections_role<WAVES, 2>(a, e, dyn_smem, hist); break;
      case 4: selections_role<WAVES, 4>(a, e, dyn_smem, hist); break;
      case 8: selections_role<WAVES, 8>(a, e, dyn_smem, hist); break;
      default: selections_role<WAVES, 16>(a, e, dyn_smem, hist); break;
    }
    return;
  }
  const int wg = blockIdx.x - a.n_sel;
  const int bh = wg / a.nsplit;
  const int sp = wg - bh * a.nsplit;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int grp = (tid >> 6) * RPW + lane / LPR;
  const int lig = lane % LPR;

  const T *Kb = static_cast<const T *>(a.Kc) + size_t(bh) * a.K * DH;
  const T *Vb = static_cast<const T *>(a.Vc) + size_t(bh) * a.K * DH;
  const int32_t *sp_row = a.slot_pos + size_t(bh) * a.K;
  const int s_ins = a.insert_slot[size_t(bh) * a.ins_stride + a.ins_off];

  float qf[EPL];
  Vec16<T>::load(static_cast<const T *>(a.q) + size_t(bh) * DH + lig * EPL, qf);
#pragma unroll
  for (int e = 0; e < EPL; ++e) qf[e] *= a.scale_log2;
  // the current token's k, v: every lane group holds them, the one that meets the reserved slot uses them
  const typename Vec16<T>::Raw kn = Vec16<T>::load_raw(static_cast<const T *>(a.k_new) + size_t(bh) * DH + lig * EPL);
  const typename Vec16<T>::Raw vn = Vec16<T>::load_raw(static_cast<const T *>(a.v_new) + size_t(bh) * DH + lig * EPL);

  const int begin = sp * a.chunk;
  const int end = min(a.K, begin + a.chunk);

  float m = -INFINITY, l = 0.f, acc[EPL];
#pragma unroll
  for (int e = 0; e < EPL; ++e) acc[e] = 0.f;

  // cache rows are read whatever they hold (no read waits for the reserved slot's index to arrive), one
  // iteration ahead of their use; the row of the reserved slot is then replaced by the current token's k, v,
  // which are also stored (the slot is marked occupied by the release kernel, which knows the reserved slot too)
  typename Vec16<T>::Raw kr[U], vr[U];
  int spv[U];
#define ATTEND_FETCH(BASE)                                                        \
  _Pragma("unroll") for (int u = 0; u < U; ++u) {                                 \
    const int slot_ = min((BASE) + u * G + grp, end - 1);                         \
    kr[u] = Vec16<T>::load_raw(Kb + size_t(slot_) * DH + lig * EPL);              \
    vr[u] = Vec16<T>::load_raw(Vb + size_t(slot_) * DH + lig * EPL);              \
    spv[u] = sp_row[slot_];                                                       \
  }
  if (begin < end) { ATTEND_FETCH(begin) }
  for (int base = begin; base < end; base += G * U) {
    float logit[U];
    bool valid[U];
    typename Vec16<T>::Raw kc[U], vc[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int slot = base + u * G + grp;
      const bool inr = slot < end;
      const bool ins = inr && slot == s_ins;
      if (ins) {
        Vec16<T>::store_raw(const_cast<T *>(Kb) + size_t(slot) * DH + lig * EPL, kn);
        Vec16<T>::store_raw(const_cast<T *>(Vb) + size_t(slot) * DH + lig * EPL, vn);
      }
      kc[u] = ins ? kn : kr[u];
      vc[u] = ins ? vn : vr[u];
      valid[u] = inr && (ins || spv[u] >= 0);
    }
    if (base + G * U < end) { ATTEND_FETCH(base + G * U) }
    float mb = m;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float dot = 0.f;
      if (valid[u]) {
        float kf[EPL];
        Vec16<T>::values(kc[u], kf);
#pragma unroll
        for (int e = 0; e < EPL; ++e) dot = fmaf(qf[e], kf[e], dot);
      }
#pragma unroll
      for (int off = LPR / 2; off > 0; off >>= 1) dot += __shfl_xor(dot, off, 64);
      logit[u] = valid[u] ? dot : -INFINITY;
      mb = fmaxf(mb, logit[u]);
      if (a.logit_out && lig == 0 && base + u * G + grp < end) a.logit_out[size_t(bh) * a.K + base + u * G + grp] = logit[u];
    }
    if (mb == -INFINITY) continue;  // nothing occupied so far in this lane group
    const float corr = exp2f(m - mb);
    l *= corr;
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[e] *= corr;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (valid[u]) {
        const float p = exp2f(logit[u] - mb);
        l += p;
        float vf[EPL];
        Vec16<T>::values(vc[u], vf);
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[e] = fmaf(p, vf[e], acc[e]);
      }
    }
    m = mb;
  }

#undef ATTEND_FETCH

  // ---- merge the G lane groups of this workgroup ----
  if (lig == 0) s_m[grp] = m;
  __syncthreads();
  float M = -INFINITY;
#pragma unroll
  for (int g = 0; g < G; ++g) M = fmaxf(M, s_m[g]);
  const float f = (m == -INFINITY) ? 0.f : exp2f(m - M);
#pragma unroll
  for (int e = 0; e < EPL; ++e) s_acc[grp][lig * EPL + e] = acc[e] * f;
  if (lig == 0) s_l[grp] = l * f;
  __syncthreads();
  if (tid < DH) {
    float sum = 0.f, L = 0.f;
#pragma unroll 8
    for (int g = 0; g < G; ++g) {
      sum += s_acc[g][tid];
      L += s_l[g];
    }
    if (a.nsplit == 1) {
      a.out[size_t(bh) * DH + tid] = sum / L;   // the current token is always present: L > 0
      if (a.ml_out && tid == 0) {
        a.ml_out[size_t(bh) * 2] = M;
        a.ml_out[size_t(bh) * 2 + 1] = L;
      }
    } else {
      float *p = a.part + (size_t(bh) * a.nsplit + sp) * (DH + 2);
      p[tid] = sum;
      if (tid == 0) {
        p[DH] = M;
        p[DH + 1] = L;
      }
    }
  }
}

template <int DH>
__global__ __launch_bounds__(DH) void attend_combine_kernel(const float *part, float *out, int nsplit, float *ml_out) {
  const int bh = blockIdx.x;
  const int tid = threadIdx.x;
  const float *p = part + size_t(bh) * nsplit * (DH + 2);
  float M = -INFINITY;
  for (int s = 0; s < nsplit; ++s) M = fmaxf(M, p[s * (DH + 2) + DH]);
  float sum = 0.f, L = 0.f;
  for (int s = 0; s < nsplit; ++s) {
    const float ms = p[s * (DH + 2) + DH];
    const float f = (ms == -INFINITY) ? 0.f : exp2f(ms - M);
    sum = fmaf(p[s * (DH + 2) + tid], f, sum);
    L = fmaf(p[s * (DH + 2) + DH + 1], f, L);
  }
  out[size_t(bh) * DH + tid] = sum / L;
  if (ml_out && tid == 0) {
    ml_out[size_t(bh) * 2] = M;
    ml_out[size_t(bh) * 2 + 1] = L;
  }
}

template <typename T, int DH>
hipError_t launch_typed(adore_ctx *ctx, const AttendArgs &a, int rows, int waves, int extra_wgs, size_t dyn_lds) {
  {
    ScopedTimer t(ctx, ADORE_KERNEL_ATTEND, ctx->stream);
    const dim3 grid(rows * a.nsplit + extra_wgs);
    if (waves == 16)
      ADORE_LAUNCH(t, (attend_kernel<T, DH, 4, 16>), grid, dim3(1024), dyn_lds, ctx->stream, a);
    else if (waves == 8)
      ADORE_LAUNCH(t, (attend_kernel<T, DH, 4, 8>), grid, dim3(512), dyn_lds, ctx->stream, a);
    else
      ADORE_LAUNCH(t, (attend_kernel<T, DH, 4, 4>), grid, dim3(256), dyn_lds, ctx->stream, a);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (a.nsplit > 1) {
    ScopedTimer t(ctx, ADORE_KERNEL_ATTEND_COMBINE, ctx->stream);
    ADORE_LAUNCH(t, (attend_combine_kernel<DH>), dim3(rows), dim3(DH), 0, ctx->stream, a.part, a.out,
                       a.nsplit, a.ml_out);
    e = hipGetLastError();
  }
  return e;
}

}  // namespace

size_t riding_lds_bytes(int n, int K, int r) {
  return size_t((n + 2) / 2) * 8 + size_t((K + 1) / 2) * 8 + ridden_choice_lds_bytes(r, n);
}

// sel: null, or the selections of this step to carry in the same launch (see SchedArgs).
hipError_t launch_attend(adore_ctx *ctx, int layer, const void *q, const void *k_new, const void *v_new,
                         float *out, const RidingSelections *sel) {
  const adore_config &c = ctx->cfg;
  const size_t layer_bytes = size_t(c.batch) * c.heads * c.cache_slots * c.head_dim * elem_size(c);
  AttendArgs a;
  a.q = q; a.k_new = k_new; a.v_new = v_new;
  a.Kc = ctx->cache_k + layer * layer_bytes;
  a.Vc = ctx->cache_v + layer * layer_bytes;
  a.slot_pos = ctx->slot_pos[ctx->cur];
  a.insert_slot = reserved_slots(ctx, ctx->cur);
  a.ins_stride = ctx->ins_stride; a.ins_off = ctx->ins_off;
  a.part = ctx->att_part;
  a.out = out;
  a.logit_out = h2o_mode(ctx) ? ctx->att_logit : nullptr;
  a.ml_out = h2o_mode(ctx) ? ctx->att_ml : nullptr;
  a.K = c.cache_slots; a.chunk = ctx->chunk; a.nsplit = ctx->nsplit;
  a.scale_log2 = 1.4426950408889634f / sqrtf(float(c.head_dim));
  const int rows = c.batch * c.heads;
  a.n_sel = 0;
  a.s.rel_wgs = 0;
  int waves = ctx->attend_waves, extra = 0;
  size_t dyn = 0;
  if (sel) {
    // 4 waves per workgroup: half of a compute unit's wave slots and registers then stay free, so the extra
    // workgroups start at once next to the attention's instead of waiting for a round of them to end
    waves = 4;
    if (const char *e = getenv("ADORE_RIDE_WAVES")) {   // tuning runs
      const int v = atoi(e);
      if (v == 4 || v == 8) waves = v;
    }
    SchedArgs &s = a.s;
    s.kpl = c.cache_slots <= 128 ? 2 : c.cache_slots <= 256 ? 4 : c.cache_slots <= 512 ? 8 : 16;
    // four heads to a wave where a row is short (four of them fit a wave's registers) and the role would otherwise
    // take more than a quarter of the chip's wave slots
    s.prio = 3;
    if (const char *e = getenv("ADORE_ROLE_PRIO")) s.prio = atoi(e);   // tuning runs
    s.hpw = s.kpl <= 4 && c.batch * c.heads > 2048 ? 4 : 1;
    if (const char *e = getenv("ADORE_RIDE_HPW")) {   // tests: the four-heads path on a small shape
      if (atoi(e) == 4 && s.kpl <= 4) s.hpw = 4;
    }
    s.rel_wgs = (c.heads - 1 + waves * s.hpw - 1) / (waves * s.hpw);
    s.slot_src = ctx->slot_pos[ctx->cur]; s.slot_dst = ctx->slot_pos[sel->dst];
    s.score = ctx->score; s.free_list = ctx->free_list[sel->dst];
    s.released_pos = ctx->released_pos; s.map_out = sel->map_out; s.rel_out = sel->rel_out;
    s.H = c.heads; s.K = c.cache_slots; s.N_max = c.max_positions; s.n = ctx->n; s.x = sel->x;
    s.R1 = c.rebuild_budget + 1;
    RebuildSelectArgs &r = s.sel;
    r.slot_pos = ctx->slot_pos[sel->dst]; r.score = ctx->score; r.free_list = ctx->free_list[sel->dst];
    r.rebuilt_pos = ctx->rebuilt_pos[sel->dst]; r.insert_slot = nullptr;
    r.map_out = sel->map_out; r.rb_out = sel->rb_out;
    r.K = c.cache_slots; r.H = c.heads; r.N_max = c.max_positions; r.n = ctx->n; r.r = sel->r;
    r.R1 = c.rebuild_budget + 1; r.Rdim = max(c.rebuild_budget, 1);
    r.words = (c.max_positions + 31) / 32;
    extra = c.batch * (s.rel_wgs + 1);
    a.n_sel = extra;
    dyn = riding_lds_bytes(ctx->n, c.cache_slots, sel->r);
  }
  if (c.dtype == ADORE_BF16) {
    return c.head_dim == 128 ? launch_typed<bf16_t, 128>(ctx, a, rows, waves, extra, dyn)
                             : launch_typed<bf16_t, 64>(ctx, a, rows, waves, extra, dyn);
  }
  return c.head_dim == 128 ? launch_typed<float, 128>(ctx, a, rows, waves, extra, dyn)
                           : launch_typed<float, 64>(ctx, a, rows, waves, extra, dyn);
}

}  // namespace adore
