// Draft-then-verify rounds (Sec. 3.1, Eq. 4-5): the batched verify pass and the round's bookkeeping.
//
// After gamma draft steps (the single-token kernels, layers 1..E + exit head) the layer-E hidden
// states of B = gamma + 1 consecutive positions go through layers E+1..N together: every weight
// matrix is streamed ONCE and multiplied with all B input vectors (B accumulators per row), which
// is what makes this schedule cheaper per token than one full pass per token.  The kernels keep
// the shape of the single-token ones (workgroups of kGBlock threads, input staged once per
// workgroup, waves looping over row-pair tasks) and, per token, the same order of operations, so a
// token's result does not depend on how many others share the pass.
#pragma once

#include "ppsd_kernels.h"

namespace ppsd {

constexpr int kMaxBatch = 5;          // gamma + 1
constexpr int kMaxGamma = kMaxBatch - 1;
constexpr int kBatchTripBlocks = kTripBlocks;   // column blocks per trip, as in the single-token kernels (4 per trip: 10-20 % slower)

// The staged vectors are written and read as whole float4 (the buffer is 16-byte aligned, a vector's
// pitch ldx and every position a multiple of 4 floats): indexing in float4 units keeps every access one
// 16-byte LDS instruction wherever the kernel is compiled.  Through a float pointer plus b * ldx the
// compiler had split the reads of the slab-walking projection into 4-byte pairs in the library build
// (38.5 us per launch at the 7B shape against 26.5 us with 16-byte reads).
__device__ __forceinline__ float4 *xs_vec(float *xs) { return reinterpret_cast<float4 *>(xs); }
__device__ __forceinline__ const float4 *xs_vec(const float *xs) { return reinterpret_cast<const float4 *>(xs); }

// RMSNorm of B vectors (vector b at x0 + b * d) into LDS xs[b * ldx + i]; same arithmetic per vector
// as NormStage.
template <typename WT, int BLOCK, int B>
struct BatchNormStage {
  float4 xv[B][kNormPer];
  float4 gv[kNormPer];
  __device__ __forceinline__ void issue(const float *x0, const float *gain, int d) {
#pragma unroll
    for (int e = 0; e < kNormPer; ++e) {
      const int i = 4 * (threadIdx.x + e * BLOCK);
      gv[e] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (i < d) gv[e] = load4_as_float(gain + i);
#pragma unroll
      for (int b = 0; b < B; ++b) {
        xv[b][e] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (i < d) xv[b][e] = load4_as_float(x0 + (size_t)b * d + i);
      }
    }
  }
  // red: B * BLOCK / 64 floats of LDS.  The B sums of squares are reduced together (one pair of barriers for
  // all of them), each in the order wg_sum takes: wave butterfly, then the waves' sums added in wave order.
  __device__ __forceinline__ void finish(int d, float eps, float *xs, int ldx, float *red) {
    constexpr int W = BLOCK / kWave;
    float ss[B];
#pragma unroll
    for (int b = 0; b < B; ++b) {
      ss[b] = 0.f;
#pragma unroll
      for (int e = 0; e < kNormPer; ++e) {
        const int i = 4 * (threadIdx.x + e * BLOCK);
        if (i < d) {
          ss[b] = fmaf(xv[b][e].x, xv[b][e].x, ss[b]); ss[b] = fmaf(xv[b][e].y, xv[b][e].y, ss[b]);
          ss[b] = fmaf(xv[b][e].z, xv[b][e].z, ss[b]); ss[b] = fmaf(xv[b][e].w, xv[b][e].w, ss[b]);
        }
      }
      ss[b] = wave_sum(ss[b]);
    }
    __syncthreads();   // red may still be read from a previous use
    if ((threadIdx.x & 63) == 0) {
#pragma unroll
      for (int b = 0; b < B; ++b) red[b * W + (threadIdx.x >> 6)] = ss[b];
    }
    __syncthreads();
#pragma unroll
    for (int b = 0; b < B; ++b) {
      float tot = 0.f;
#pragma unroll
      for (int w = 0; w < W; ++w) tot += red[b * W + w];
      const float rs = 1.0f / sqrtf(tot / (float)d + eps);
#pragma unroll
      for (int e = 0; e < kNormPer; ++e) {
        const int i = 4 * (threadIdx.x + e * BLOCK);
        if (i < d)
          xs_vec(xs)[b * (ldx >> 2) + (xs_pos<WT>(i) >> 2)] = make_float4(xv[b][e].x * rs * gv[e].x, xv[b][e].y * rs * gv[e].y,
                                                                           xv[b][e].z * rs * gv[e].z, xv[b][e].w * rs * gv[e].w);
      }
    }
    __syncthreads();
  }
};

// One trip of weights against B staged vectors.  Per (row, vector) the products are added in the
// same order as in trip_consume.
template <typename WT, int B>
__device__ __forceinline__ void trip_consume_b(const Trip<WT, kTripRows, kBatchTripBlocks> &t, const float *xs, int ldx,
                                               int cb, int C, float (&acc)[kTripRows][B]) {
  constexpr int N = Pack<WT>::N;
  constexpr int kStride = kWave * N;
  const int lane = threadIdx.x & 63;
#pragma unroll
  for (int k = 0; k < kBatchTripBlocks; ++k) {
    const int c = (cb + k) * kStride + lane * N;
    if (c < C) {
      float w0[N], w1[N];
      Pack<WT>::unpack(t.u[0 * kBatchTripBlocks + k], w0);
      Pack<WT>::unpack(t.u[1 * kBatchTripBlocks + k], w1);
#pragma unroll
      for (int b = 0; b < B; ++b) {
        float x[N];
#pragma unroll
        for (int q = 0; q < N / 4; ++q) {
          const float4 v = xs_vec(xs)[b * (ldx >> 2) + (cb + k) * (kStride >> 2) + q * kWave + lane];
          x[4 * q] = v.x; x[4 * q + 1] = v.y; x[4 * q + 2] = v.z; x[4 * q + 3] = v.w;
        }
#pragma unroll
        for (int e = 0; e < N; ++e) acc[0][b] = fmaf(w0[e], x[e], acc[0][b]);
#pragma unroll
        for (int e = 0; e < N; ++e) acc[1][b] = fmaf(w1[e], x[e], acc[1][b]);
      }
    }
  }
}

// gemv_tasks with B right-hand sides: epi(task, s) with s[row][vector].
template <typename WT, int B, typename RowsFn, typename EpiFn>
__device__ __forceinline__ void gemv_tasks_b(Trip<WT, kTripRows, kBatchTripBlocks> &trip, const WT *(&rows)[kTripRows],
                                             int task, int n_tasks, int tw, int C, const float *xs, int ldx,
                                             RowsFn &&set_rows, EpiFn &&epi) {
  const int nblk = col_blocks<WT>(C);
  while (task < n_tasks) {
    float acc[kTripRows][B];
#pragma unroll
    for (int r = 0; r < kTripRows; ++r)
#pragma unroll
      for (int b = 0; b < B; ++b) acc[r][b] = 0.f;
    const int next = task + tw;
    for (int cb = 0; cb < nblk; cb += kBatchTripBlocks) {
      trip_consume_b<WT, B>(trip, xs, ldx, cb, C, acc);
      if (cb + kBatchTripBlocks < nblk) {
        trip_load<WT, kTripRows, kBatchTripBlocks>(trip, rows, cb + kBatchTripBlocks, nblk, C);
      } else if (next < n_tasks) {
        set_rows(next);
        trip_load<WT, kTripRows, kBatchTripBlocks>(trip, rows, 0, nblk, C);
      }
    }
    float s[kTripRows][B];
#pragma unroll
    for (int r = 0; r < kTripRows; ++r)
#pragma unroll
      for (int b = 0; b < B; ++b) s[r][b] = wave_sum(acc[r][b]);
    epi(task, s);
    task = next;
  }
}

// ------------------------------------------------------------------------------------------
// RMSNorm + QKV + rotary + KV append for B tokens at positions pos .. pos + B - 1.
// x_slot0: residual slot of token 0 (tokens are in consecutive slots).  Dynamic LDS = B * d floats.
template <typename WT, int B>
__global__ __launch_bounds__(kGBlock) void k_qkv_b(Common c, int layer, int x_slot0, const float *gain, const WT *wqkv,
                                                   float *qout) {
  extern __shared__ __align__(16) float xs[];
  __shared__ float red[kGWaves * B];
  const Dims &m = c.dm;
  const int d = m.d;
  BatchNormStage<WT, kGBlock, B> in;
  in.issue(c.xbuf + (size_t)x_slot0 * d, gain, d);
  const StageIn si = stage_in(c, kEesdVerify);
  if (!si.active) return;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int half = m.hd >> 1;
  const int n_tasks = (m.n_h + 2 * m.n_kv) * half;
  const int gw = blockIdx.x * kGWaves + wave, tw = gridDim.x * kGWaves;
  const int nq = m.n_h * m.hd;
  const WT *rows[kTripRows];
  auto set_rows = [&](int task) {
    const int head = task / half, i = task - head * half;
    rows[0] = wqkv + (size_t)(head * m.hd + i) * d;
    rows[1] = rows[0] + (size_t)half * d;
  };
  Trip<WT, kTripRows, kBatchTripBlocks> trip;
  if (gw < n_tasks) { set_rows(gw); trip_load<WT, kTripRows, kBatchTripBlocks>(trip, rows, 0, col_blocks<WT>(d), d); }
  const int ldx = xs_floats((int)sizeof(WT), d);
  in.finish(d, m.eps, xs, ldx, red);
  gemv_tasks_b<WT, B>(trip, rows, gw, n_tasks, tw, d, xs, ldx, set_rows, [&](int task, float (&s)[kTripRows][B]) {
    if (lane != 0) return;
    const int h = task / half, i = task - h * half;
#pragma unroll
    for (int b = 0; b < B; ++b) {
      const int pos = si.pos + b;
      float lo = s[0][b], hi = s[1][b];
      if (h < m.n_h + m.n_kv) {
        const float cs = c.rope_cos[(size_t)pos * half + i];
        const float sn = c.rope_sin[(size_t)pos * half + i];
        const float rlo = lo * cs - hi * sn;
        const float rhi = hi * cs + lo * sn;
        lo = rlo; hi = rhi;
      }
      if (h < m.n_h) {
        qout[(size_t)b * nq + h * m.hd + i] = lo;
        qout[(size_t)b * nq + h * m.hd + i + half] = hi;
      } else {
        const int which = (h < m.n_h + m.n_kv) ? 0 : 1;
        const int kvh = which ? h - m.n_h - m.n_kv : h - m.n_h;
        WT *dst = kv_row<WT>(c, c.page_table, layer, pos, kvh, which);
        dst[i] = Pack<WT>::from_float(lo);
        dst[i + half] = Pack<WT>::from_float(hi);
      }
    }
  });
}

// Attention of B queries: grid = (n_kv, n_splits, B); query b sits at position pos + b and sees the
// rows up to its own (the B rows of this pass were appended by k_qkv_b just before).
template <typename WT, int HD, int G>
__global__ __launch_bounds__(kGBlock) void k_attn_b(Common c, int layer, const float *q, float *aout, float *partials,
                                                    int *counters) {
  constexpr int GPB = kGBlock / (HD / Pack<WT>::N);
  // one record per wave and query head (the groups of a wave are merged through shuffles first); the merge of
  // the splits reuses it for 3 * G * kMaxAttnSplits floats
  __shared__ float merge[(kGBlock / kWave) * G * (HD + 2)];
  static_assert((kGBlock / kWave) * (HD + 2) >= 3 * kMaxAttnSplits, "the split merge's arrays fit the records");
  __shared__ int s_last;
  __shared__ int32_t s_ptab[kAttnLdsPages];
  const bool lds_pt = c.dm.n_pages <= kAttnLdsPages;
  if (lds_pt)
    for (int i = threadIdx.x; i < c.dm.n_pages; i += kGBlock) s_ptab[i] = c.page_table[i];
  const StageIn si = stage_in(c, kEesdVerify);
  if (!si.active) return;
  __syncthreads();
  const int b = blockIdx.z;
  const int nq = c.dm.n_h * HD;
  float *part_b = partials + (size_t)b * c.dm.n_h * gridDim.y * (HD + 2);
  int *count_b = counters + (size_t)b * c.dm.n_kv * kCounterStride;
  // one call per address space of the page table (a selected pointer would turn the lookups into flat loads)
  if (lds_pt)
    attn_unit<WT, HD, G, kGBlock>(c, s_ptab, layer, si.pos + b, blockIdx.x, blockIdx.y, gridDim.y, q + (size_t)b * nq,
                                  aout + (size_t)b * nq, part_b, count_b, merge, &s_last);
  else
    attn_unit<WT, HD, G, kGBlock>(c, c.page_table, layer, si.pos + b, blockIdx.x, blockIdx.y, gridDim.y, q + (size_t)b * nq,
                                  aout + (size_t)b * nq, part_b, count_b, merge, &s_last);
}

// out_b[r] = resid_b[r] + W[r, c0 : c0 + Cs] . vin_b[c0 : c0 + Cs] for B tokens; vin is [B][C_total].
// A matrix whose B staged input vectors exceed the LDS budget is processed in column slabs by
// consecutive launches (the later ones with resid = out).  Dynamic LDS = B * Cs floats.
template <typename WT, int B>
__global__ __launch_bounds__(kGBlock) void k_proj_resid_b(Common c, const float *vin, int C_total, int c0, int Cs,
                                                          const WT *W, int n_rows, int resid_slot0, int out_slot0) {
  extern __shared__ __align__(16) float xs[];
  const StageIn si = stage_in(c, kEesdVerify);
  if (!si.active) return;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int n_tasks = (n_rows + 1) >> 1;
  const int gw = blockIdx.x * kGWaves + wave, tw = gridDim.x * kGWaves;
  const WT *rows[kTripRows];
  auto set_rows = [&](int task) {
    rows[0] = W + (size_t)(2 * task) * C_total + c0;
    rows[1] = W + (size_t)min(2 * task + 1, n_rows - 1) * C_total + c0;
  };
  Trip<WT, kTripRows, kBatchTripBlocks> trip;
  if (gw < n_tasks) { set_rows(gw); trip_load<WT, kTripRows, kBatchTripBlocks>(trip, rows, 0, col_blocks<WT>(Cs), Cs); }
  const int ldx = xs_floats((int)sizeof(WT), Cs);
#pragma unroll
  for (int b = 0; b < B; ++b)
    for (int i = 4 * threadIdx.x; i < Cs; i += 4 * kGBlock)
      xs_vec(xs)[b * (ldx >> 2) + (xs_pos<WT>(i) >> 2)] = *(const float4 *)(vin + (size_t)b * C_total + c0 + i);
  __syncthreads();
  const int d = c.dm.d;
  const float *resid = c.xbuf + (size_t)resid_slot0 * d;
  float *out = c.xbuf + (size_t)out_slot0 * d;
  gemv_tasks_b<WT, B>(trip, rows, gw, n_tasks, tw, Cs, xs, ldx, set_rows, [&](int task, float (&s)[kTripRows][B]) {
    const int r = 2 * task + lane;
    if (lane < 2 && r < n_rows) {
#pragma unroll
      for (int b = 0; b < B; ++b) out[(size_t)b * d + r] = resid[(size_t)b * d + r] + (lane == 0 ? s[0][b] : s[1][b]);
    }
  });
}

// The same projection when the B staged input vectors exceed the LDS budget: one launch, one row per wave
// (n_rows waves in all), the column slabs taken in turn inside the kernel.  A wave keeps its row's B sums in
// registers across the slabs, so per (row, token) the products are added in exactly the order of the
// single-token kernel, and the first weight loads of a slab are in flight while the slab's inputs are staged.
// Cs: columns per slab, a multiple of a column block (64 lanes x 16 bytes).  Dynamic LDS = B * Cs floats.
// grid = ceil(n_rows / waves per workgroup).
template <typename WT, int B>
__global__ __launch_bounds__(kGBlock) void k_proj_resid_bs(Common c, const float *vin, int C, int Cs, const WT *W, int n_rows,
                                                           int resid_slot0, int out_slot0) {
  extern __shared__ __align__(16) float xs[];
  constexpr int N = Pack<WT>::N, KB = kProjTripBlocks, kStride = kWave * N;
  const StageIn si = stage_in(c, kEesdVerify);
  if (!si.active) return;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int row = blockIdx.x * kGWaves + wave;
  const bool mine = row < n_rows;                        // every wave takes part in the barriers
  const WT *rows[1] = {W + (size_t)(mine ? row : 0) * C};
  Trip<WT, 1, KB> trip;
  {
    const int w0 = C < Cs ? C : Cs;
    if (mine) trip_load<WT, 1, KB>(trip, rows, 0, col_blocks<WT>(w0), w0);
  }
  float acc[B];
#pragma unroll
  for (int b = 0; b < B; ++b) acc[b] = 0.f;
  const int ldx = xs_floats((int)sizeof(WT), Cs);
  for (int c0 = 0; c0 < C; c0 += Cs) {
    const int w = C - c0 < Cs ? C - c0 : Cs, nblk = col_blocks<WT>(w);
    if (c0 > 0) __syncthreads();                         // the slab before has been read
#pragma unroll
    for (int b = 0; b < B; ++b)
      for (int i = 4 * threadIdx.x; i < w; i += 4 * kGBlock)
        xs_vec(xs)[b * (ldx >> 2) + (xs_pos<WT>(i) >> 2)] = *(const float4 *)(vin + (size_t)b * C + c0 + i);
    __syncthreads();
    if (mine) {
      for (int cb = 0; cb < nblk; cb += KB) {
#pragma unroll
        for (int k = 0; k < KB; ++k) {
          if ((cb + k) * kStride + lane * N < w) {
            float wf[N];
            Pack<WT>::unpack(trip.u[k], wf);
#pragma unroll
            for (int b = 0; b < B; ++b) {
              float x[N];
#pragma unroll
              for (int q = 0; q < N / 4; ++q) {
                const float4 v = xs_vec(xs)[b * (ldx >> 2) + (cb + k) * (kStride >> 2) + q * kWave + lane];
                x[4 * q] = v.x; x[4 * q + 1] = v.y; x[4 * q + 2] = v.z; x[4 * q + 3] = v.w;
              }
#pragma unroll
              for (int e = 0; e < N; ++e) acc[b] = fmaf(wf[e], x[e], acc[b]);
            }
          }
        }
        if (cb + KB < nblk) {
          trip_load<WT, 1, KB>(trip, rows, cb + KB, nblk, w);
        } else if (c0 + Cs < C) {                        // first trip of the next slab
          const int w2 = C - c0 - Cs < Cs ? C - c0 - Cs : Cs;
          rows[0] += Cs;
          trip_load<WT, 1, KB>(trip, rows, 0, col_blocks<WT>(w2), w2);
        }
      }
    }
  }
  if (!mine) return;
  const int d = c.dm.d;
  const float *resid = c.xbuf + (size_t)resid_slot0 * d;
  float *out = c.xbuf + (size_t)out_slot0 * d;
#pragma unroll
  for (int b = 0; b < B; ++b) {
    const float sum = wave_sum(acc[b]);
    if (lane == 0) out[(size_t)b * d + row] = resid[(size_t)b * d + row] + sum;
  }
}

// RMSNorm + gate/up + SwiGLU for B tokens: mout is [B][f].  Dynamic LDS = B * d floats.
template <typename WT, int B>
__global__ __launch_bounds__(kGBlock) void k_gate_up_b(Common c, int x_slot0, const float *gain, const WT *wgu,
                                                       float *mout) {
  extern __shared__ __align__(16) float xs[];
  __shared__ float red[kGWaves * B];
  const Dims &m = c.dm;
  const int d = m.d, f = m.f;
  BatchNormStage<WT, kGBlock, B> in;
  in.issue(c.xbuf + (size_t)x_slot0 * d, gain, d);
  const StageIn si = stage_in(c, kEesdVerify);
  if (!si.active) return;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int gw = blockIdx.x * kGWaves + wave, tw = gridDim.x * kGWaves;
  const WT *rows[kTripRows];
  auto set_rows = [&](int task) {
    rows[0] = wgu + (size_t)task * d;
    rows[1] = wgu + (size_t)(f + task) * d;
  };
  Trip<WT, kTripRows, kBatchTripBlocks> trip;
  if (gw < f) { set_rows(gw); trip_load<WT, kTripRows, kBatchTripBlocks>(trip, rows, 0, col_blocks<WT>(d), d); }
  const int ldx = xs_floats((int)sizeof(WT), d);
  in.finish(d, m.eps, xs, ldx, red);
  gemv_tasks_b<WT, B>(trip, rows, gw, f, tw, d, xs, ldx, set_rows, [&](int task, float (&s)[kTripRows][B]) {
    if (lane != 0) return;
#pragma unroll
    for (int b = 0; b < B; ++b) {
      const float g = s[0][b], u = s[1][b];
      mout[(size_t)b * f + task] = g / (1.0f + __expf(-g)) * u;
    }
  });
}

// LM head of B tokens: one (value, index) candidate per workgroup and token in
// cand[b * kMaxWorkgroups + blockIdx.x].  Logit rows (parity harness): row = tokens committed so far + b;
// logits_out != nullptr receives all logits as [B][V].
template <typename WT, int B>
__global__ __launch_bounds__(kGBlock) void k_head_b(Common c, int x_slot0, const float *gain, const WT *W, float2 *cand,
                                                    float *logits_log, float *logits_out) {
  extern __shared__ __align__(16) float xs[];
  __shared__ float red[kGWaves * B];
  __shared__ float bv[kGWaves][B];
  __shared__ int bi[kGWaves][B];
  const Dims &m = c.dm;
  const int d = m.d, V = m.V;
  BatchNormStage<WT, kGBlock, B> in;
  in.issue(c.xbuf + (size_t)x_slot0 * d, gain, d);
  const StageIn si = stage_in(c, kEesdVerify);
  if (!si.active) return;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int n_tasks = (V + 1) >> 1;
  const int gw = blockIdx.x * kGWaves + wave, tw = gridDim.x * kGWaves;
  const WT *rows[kTripRows];
  auto set_rows = [&](int task) {
    rows[0] = W + (size_t)(2 * task) * d;
    rows[1] = W + (size_t)min(2 * task + 1, V - 1) * d;
  };
  Trip<WT, kTripRows, kBatchTripBlocks> trip;
  if (gw < n_tasks) { set_rows(gw); trip_load<WT, kTripRows, kBatchTripBlocks>(trip, rows, 0, col_blocks<WT>(d), d); }
  const int ldx = xs_floats((int)sizeof(WT), d);
  in.finish(d, m.eps, xs, ldx, red);
  const int row0 = c.st->gen_count;
  float best[B];
  int besti[B];
#pragma unroll
  for (int b = 0; b < B; ++b) { best[b] = -INFINITY; besti[b] = kNoIndex; }
  gemv_tasks_b<WT, B>(trip, rows, gw, n_tasks, tw, d, xs, ldx, set_rows, [&](int task, float (&s)[kTripRows][B]) {
    const int r = 2 * task;
#pragma unroll
    for (int b = 0; b < B; ++b) {
      if (better(s[0][b], r, best[b], besti[b])) { best[b] = s[0][b]; besti[b] = r; }
      if (r + 1 < V && better(s[1][b], r + 1, best[b], besti[b])) { best[b] = s[1][b]; besti[b] = r + 1; }
      if (logits_log && lane == 0 && row0 + b < m.debug_rows) {
        float *lrow = logits_log + (size_t)(row0 + b) * V;
        lrow[r] = s[0][b];
        if (r + 1 < V) lrow[r + 1] = s[1][b];
      }
      if (logits_out && lane == 0) {           // sampling needs the whole distribution of every token
        logits_out[(size_t)b * V + r] = s[0][b];
        if (r + 1 < V) logits_out[(size_t)b * V + r + 1] = s[1][b];
      }
    }
  });
  if (lane == 0) {
#pragma unroll
    for (int b = 0; b < B; ++b) { bv[wave][b] = best[b]; bi[wave][b] = besti[b]; }
  }
  __syncthreads();
  if (threadIdx.x < B) {
    const int b = threadIdx.x;
    float v = bv[0][b];
    int ix = bi[0][b];
    for (int w = 1; w < kGWaves; ++w)
      if (better(bv[w][b], bi[w][b], v, ix)) { v = bv[w][b]; ix = bi[w][b]; }
    cand[(size_t)b * kMaxWorkgroups + blockIdx.x] = make_float2(v, __int_as_float(ix));
  }
}

// After draft step j: finish the exit head's argmax and make it the token of draft step j + 1.
__global__ __launch_bounds__(kBlock) void k_eesd_pick(Common c, const float2 *cand_exit, int j) {
  __shared__ float sv[kWavesPerBlock];
  __shared__ int si_[kWavesPerBlock];
  DevState *st = c.st;
  if (!(st->n_out < st->target)) return;
  const int tok = reduce_candidates<kBlock>(cand_exit, c.dm.head_blocks, c.dm.V, sv, si_);
  if (threadIdx.x == 0) st->ee_draft[j + 1] = tok;
}

// Stochastic rounds (Sec. 3.1, Eq. 1-2 as stated: gamma sampled drafts, checked in order).
// After draft step j: p_j = softmax(exit logits / T) is kept in probs_e[j] and draft x_{j+1} ~ p_j
// becomes the token of step j + 1.
__global__ __launch_bounds__(kSBlock) void k_eesd_pick_sample(Common c, const float *logits_exit, float *probs_e, int j,
                                                              float inv_temp, uint32_t seed) {
  __shared__ float scan[kSBlock + 1];
  __shared__ float buf[kSWaves];
  __shared__ int s_pick;
  DevState *st = c.st;
  if (!(st->n_out < st->target)) return;
  const int V = c.dm.V;
  float m = -INFINITY;
  for (int i = threadIdx.x; i < V; i += kSBlock) m = fmaxf(m, logits_exit[i]);
  const float mp = sblock_max(m, buf);
  float sp;
  const int d = sample_index([&](int i) { return __expf((logits_exit[i] - mp) * inv_temp); }, V,
                             uniform24(seed, st->t + j + 1, kPurDraft), scan, &s_pick, &sp);
  float *pj = probs_e + (size_t)j * V;
  for (int i = threadIdx.x; i < V; i += kSBlock) pj[i] = __expf((logits_exit[i] - mp) * inv_temp) / sp;
  if (threadIdx.x == 0) st->ee_draft[j + 1] = d;
}

// End of a stochastic round.  logits_b: [gamma + 1][V] from the batched LM head (row j: the full
// model's logits for position t + j + 1).  Draft x_{j+1} is accepted iff u * p_j(x) <= q_j(x); the
// first rejected one is replaced by a token from max(0, q_j - p_j); if all are accepted one more
// token is sampled from q_gamma.  Commit and rollback as in the greedy round.
__global__ __launch_bounds__(kSBlock) void k_eesd_commit_sample(Common c, const float *logits_b, const float *probs_e,
                                                                int32_t *out_tokens, int32_t *drafts_log, int gamma,
                                                                float inv_temp, uint32_t seed) {
  __shared__ float scan[kSBlock + 1];
  __shared__ float buf[kSWaves];
  __shared__ int s_pick;
  __shared__ int s_tok[kMaxBatch];
  DevState *st = c.st;
  if (!(st->n_out < st->target)) return;
  const int V = c.dm.V;
  const int t = st->t;
  int n = 0;
  bool stopped = false;
  while (n < gamma && !stopped) {
    const float *lg = logits_b + (size_t)n * V;
    const float *pj = probs_e + (size_t)n * V;
    const int pos = t + n + 1;
    const int d = st->ee_draft[n + 1];
    float m = -INFINITY;
    for (int i = threadIdx.x; i < V; i += kSBlock) m = fmaxf(m, lg[i]);
    const float mq = sblock_max(m, buf);
    float sq;
    (void)sample_index([&](int i) { return __expf((lg[i] - mq) * inv_temp); }, V, 0.f, scan, &s_pick, &sq);
    const float qd = __expf((lg[d] - mq) * inv_temp) / sq;
    const bool ok = uniform24(seed, pos, kPurAccept) * pj[d] <= qd;
    int tok = d;
    if (!ok) {
      auto resid = [&](int i) { return fmaxf(0.f, __expf((lg[i] - mq) * inv_temp) / sq - pj[i]); };
      float sr;
      tok = sample_index(resid, V, uniform24(seed, pos, kPurResample), scan, &s_pick, &sr);
      if (!(sr > 0.f))
        tok = sample_index([&](int i) { return __expf((lg[i] - mq) * inv_temp); }, V, uniform24(seed, pos, kPurResample),
                           scan, &s_pick, nullptr);
      stopped = true;
    }
    if (threadIdx.x == 0) s_tok[n] = tok;
    if (ok) ++n;
  }
  if (n == gamma) {                             // every draft accepted: the full model's own token follows
    const float *lg = logits_b + (size_t)gamma * V;
    float m = -INFINITY;
    for (int i = threadIdx.x; i < V; i += kSBlock) m = fmaxf(m, lg[i]);
    const float mq = sblock_max(m, buf);
    const int tok = sample_index([&](int i) { return __expf((lg[i] - mq) * inv_temp); }, V,
                                 uniform24(seed, t + gamma + 1, kPurVanilla), scan, &s_pick, nullptr);
    if (threadIdx.x == 0) s_tok[gamma] = tok;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    st->stats[11] += 1;
    st->stats[1] += n + 1 < gamma ? n + 1 : gamma;
    st->stats[2] += n;
    if (n < gamma) { st->stats[3] += 1; st->stats[6] += 1; }
    const int room = st->target - st->n_out;
    const int k = n + 1 < room ? n + 1 : room;
    for (int i = 0; i < k; ++i) {
      out_tokens[st->n_out + i] = s_tok[i];
      drafts_log[st->gen_count + i] = i < gamma ? st->ee_draft[i + 1] : -1;
    }
    st->n_out += k; st->gen_count += k; st->stats[0] += k;
    st->t += k;
    st->last_token = s_tok[k - 1];
  }
}

// End of a round: the full model's tokens v_0..v_gamma, the accepted prefix, the commit.
// Drafts x_1..x_gamma are in ee_draft[1..gamma]; v_j belongs to position t + j + 1.  The n leading
// drafts equal to their v are accepted and v_0..v_n committed (cut at the call's target: what
// lies beyond is discarded and drafted again).  Rows of rejected drafts are dropped by not
// advancing past them: the next round rewrites those positions before reading them.
__global__ __launch_bounds__(kBlock) void k_eesd_commit(Common c, const float2 *cand_b, int32_t *out_tokens,
                                                        int32_t *drafts_log, int gamma) {
  __shared__ float sv[kWavesPerBlock];
  __shared__ int si_[kWavesPerBlock];
  DevState *st = c.st;
  if (!(st->n_out < st->target)) return;
  int v[kMaxBatch];
  for (int b = 0; b <= gamma; ++b) v[b] = reduce_candidates<kBlock>(cand_b + (size_t)b * kMaxWorkgroups, c.dm.head_blocks, c.dm.V, sv, si_);
  if (threadIdx.x == 0) {
    int n = 0;
    while (n < gamma && st->ee_draft[n + 1] == v[n]) ++n;
    st->stats[11] += 1;                         // rounds
    st->stats[1] += n + 1 < gamma ? n + 1 : gamma;   // drafts compared: up to and including the first mismatch
    st->stats[2] += n;
    if (n < gamma) { st->stats[3] += 1; st->stats[6] += 1; }
    const int room = st->target - st->n_out;
    const int k = n + 1 < room ? n + 1 : room;
    for (int i = 0; i < k; ++i) {
      out_tokens[st->n_out + i] = v[i];
      drafts_log[st->gen_count + i] = i < gamma ? st->ee_draft[i + 1] : -1;
    }
    st->n_out += k; st->gen_count += k; st->stats[0] += k;
    st->t += k;
    st->last_token = v[k - 1];
  }
}

}  // namespace ppsd
