// Decode-step kernels (steps a1..a10 of one PPSD step), gfx950, wave64.
//
// Every kernel starts by resolving its stage's input from the device state (stage_in); a stage
// with nothing to do returns at once, so the host can enqueue steps without knowing accept/reject
// outcomes.
//
// The four weight-streaming kernels (k_qkv, k_proj_resid, k_gate_up, k_head) share one shape:
// workgroups of kGBlock threads, a few per CU, each staging the input vector ONCE and every wave
// looping over row-pair tasks with a stride of the whole grid (gemv_tasks).  Staging per small
// workgroup was measured to cost ~8 us per kernel: a late workgroup's input loads queue behind
// the weight loads already streaming through its CU.
#pragma once

#include "ppsd_device.h"

namespace ppsd {

// Launch policy of the weight-streaming kernels: one wave per row-pair task up to a few workgroups
// per CU, beyond that the waves loop.
constexpr int kGemvWgsPerCu = 3;       // what stays resident: the kernels take 72-80 VGPRs, 6 waves per SIMD
constexpr int kGateUpWgsPerCu = 2;
constexpr int kMaxWorkgroups = 1024;   // also the capacity of the head-candidate arrays
// Every wave gets the same number k of tasks (the last ones one fewer at most): k = the smallest
// count with which all workgroups are resident at once, grid = just enough workgroups for k tasks
// per wave.  A grid of "capacity" workgroups leaves part of the waves with one task more than the
// others (gate/up on 512 workgroups: 2.69 tasks per wave, a third of the run at 2/3 occupancy).
inline int gemv_grid_for(int n_tasks, int n_cu, int wgs_per_cu) {
  int cap = wgs_per_cu * n_cu;
  if (cap > kMaxWorkgroups) cap = kMaxWorkgroups;
  const int k = (n_tasks + cap * kGWaves - 1) / (cap * kGWaves);
  const int grid = (n_tasks + kGWaves * k - 1) / (kGWaves * k);
  return grid < 1 ? 1 : grid;
}

// KV pool addressing: [layer][physical page][kv head][K=0 / V=1][slot][hd]
// ptab: the page table, in global memory or a copy in LDS.
template <typename WT>
__device__ __forceinline__ WT *kv_row(const Common &c, const int32_t *ptab, int layer, int pos, int kvh, int which) {
  const Dims &m = c.dm;
  // page sizes are powers of two: shifts instead of a division per row; the block index fits 32 bits
  // (layers x pages x KV heads x 2 < 2^31 at any supported size)
  const int page = ptab[pos >> m.page_shift];
  const int slot = pos & (m.page_tokens - 1);
  const uint32_t block = (((uint32_t)layer * m.n_pages + page) * m.n_kv + kvh) * 2 + which;
  const size_t idx = ((size_t)block << m.page_shift) + slot;
  return (WT *)c.kv_pool + idx * m.hd;
}

// ------------------------------------------------------------------------------------------
// a1-a3: (embedding) + RMSNorm + QKV GEMV + rotary + KV append.
// A task is the row pair (i, i + hd/2) of one head, so the rotation partner is local to the wave.
template <typename WT, int DEPTH>
__global__ __launch_bounds__(kGBlock) void k_qkv(Common c, int role, int layer, int xin_sel, int from_embed,
                                                 const WT *embed, const float *gain, const WT *wqkv,
                                                 float *qout) {
  extern __shared__ __align__(16) float xs[];
  __shared__ float red[kGWaves];
  const Dims &m = c.dm;
  const int d = m.d;
  NormStage<WT, kGBlock> in;
  const bool early = !from_embed && static_slot(xin_sel);
  if (early) in.issue(c.xbuf + (size_t)xin_sel * d, (const WT *)nullptr, gain, d);   // under the state read
  const StageIn si = stage_in(c, role);
  if (!si.active) return;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int half = m.hd >> 1;
  const int n_tasks = (m.n_h + 2 * m.n_kv) * half;
  const int nwg = active_workgroups(c, role);
  if ((int)blockIdx.x >= nwg) return;
  const int gw = blockIdx.x * kGWaves + wave, tw = nwg * kGWaves;

  const WT *rows[kTripRows];
  auto set_rows = [&](int task) {
    const int head = task / half, i = task - head * half;
    rows[0] = wqkv + (size_t)(head * m.hd + i) * d;
    rows[1] = rows[0] + (size_t)half * d;
  };
  Trips<WT, kTripRows, kTripBlocks, DEPTH> trips;
  if (!early) {
    const WT *xrow = from_embed ? embed + (size_t)si.tok * d : nullptr;
    in.issue(from_embed ? nullptr : xslot(c, xin_sel), xrow, gain, d);
  }
  trips.start(rows, gw, n_tasks, tw, d, set_rows);
  in.finish(d, m.eps, xs, red, (from_embed && blockIdx.x == 0) ? xslot(c, xin_sel) : nullptr);
  trips.run(rows, gw, n_tasks, tw, d, xs, set_rows, [&](int task, const float (&sum)[kTripRows]) {
    if (lane != 0) return;
    float lo = sum[0], hi = sum[1];
    const int h = task / half, i = task - h * half;
    if (h < m.n_h + m.n_kv) {   // q or k head: rotate the pair by the position angle
      const float cs = c.rope_cos[(size_t)si.pos * half + i];
      const float sn = c.rope_sin[(size_t)si.pos * half + i];
      const float rlo = lo * cs - hi * sn;
      const float rhi = hi * cs + lo * sn;
      lo = rlo; hi = rhi;
    }
    if (h < m.n_h) {
      qout[h * m.hd + i] = lo;
      qout[h * m.hd + i + half] = hi;
    } else {
      const int which = (h < m.n_h + m.n_kv) ? 0 : 1;
      const int kvh = which ? h - m.n_h - m.n_kv : h - m.n_h;
      WT *dst = kv_row<WT>(c, c.page_table, layer, si.pos, kvh, which);
      dst[i] = Pack<WT>::from_float(lo);
      dst[i + half] = Pack<WT>::from_float(hi);
    }
  });
}

// ------------------------------------------------------------------------------------------
// a4: decode attention over the paged KV cache, one (KV head, split) unit per call.
// A group of GS = HD / N lanes owns one position at a time (each lane holds N consecutive dims of
// the K and V rows, loaded as one 16-byte vector); the G query heads that share this KV head reuse
// the same K/V registers.  Every group keeps a running softmax (max, sum, weighted V) and the
// groups are merged through LDS (`merge`, BLOCK/GS * G * (HD+2) floats) in a fixed order.  With
// several splits the last workgroup to finish a KV head merges the splits, also in fixed order.
// Must be called by all BLOCK threads of the workgroup; ends with the workgroup synchronised.
constexpr int kCounterStride = 64;   // ints between the arrival counters of two KV heads: atomics on one
                                    // cache line serialise, each head gets a line of its own
constexpr int kMergeBatch = 32;   // splits whose partial results the merging workgroup loads at once
constexpr int kMaxAttnSplits = 64; // splits along the sequence, at most (G * splits <= threads of the workgroup)
template <typename WT, int HD, int G, int BLOCK>
__device__ __forceinline__ void attn_unit(const Common &c, const int32_t *ptab, int layer, int pos, int kvh,
                                          int split, int n_splits, const float *q, float *aout, float *partials,
                                          int *counters, float *merge, int *s_last) {
  constexpr int N = Pack<WT>::N;
  constexpr int GS = HD / N;               // lanes per position
  constexpr int GPB = BLOCK / GS;          // position groups per workgroup
  constexpr int REC = HD + 2;              // m, l, acc[HD]
  const Dims &m = c.dm;
  const int len = pos + 1;
  // split ranges are page aligned
  int chunk = (len + n_splits - 1) / n_splits;
  chunk = ((chunk + m.page_tokens - 1) / m.page_tokens) * m.page_tokens;
  const int start = split * chunk;
  const int end = min(len, start + chunk);

  const int tid = threadIdx.x;
  const int grp = tid / GS, j = tid % GS;

  float qr[G][N];
#pragma unroll
  for (int g = 0; g < G; ++g)
#pragma unroll
    for (int k = 0; k < N; ++k) qr[g][k] = q[(kvh * G + g) * HD + j * N + k] * m.qscale;

  float mx[G], l[G], acc[G][N];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    mx[g] = kNegBig; l[g] = 0.f;
#pragma unroll
    for (int k = 0; k < N; ++k) acc[g][k] = 0.f;
  }

  // A block = U positions per group (U * GPB per workgroup).  The next block's K/V rows are loaded
  // before the current block is used, so a wave's arithmetic runs under its own loads; within a
  // block the running maximum is raised once and the accumulators rescaled once.
  constexpr int U = 2;   // (4: a split of 272 positions pads to 384 instead of 320, and four query heads per KV head need 158 VGPRs instead of 124)
  uint4 ku[U], vu[U], kn[U], vn[U];
  auto load_block = [&](int p0, uint4 (&kk)[U], uint4 (&vv)[U]) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int p = p0 + u * GPB;
      const int pc = p < end ? p : (p0 < end ? p0 : start);     // an in-range row; its result is masked out
      const WT *kr = kv_row<WT>(c, ptab, layer, pc, kvh, 0) + j * N;
      kk[u] = *(const uint4 *)kr;
      vv[u] = *(const uint4 *)(kr + (size_t)m.page_tokens * HD);
    }
  };
  auto process = [&](int p0, const uint4 (&kk)[U], const uint4 (&vv)[U]) {
    // positions p0 + u * GPB; a whole u-slice of the split's last block may lie behind its end (the same for
    // every group of the workgroup): its arithmetic is skipped, the result is the same
    const int b0 = p0 - grp;
    float sc[G][U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (b0 + u * GPB < end) {
        float kf[N];
        Pack<WT>::unpack(kk[u], kf);
        const bool ok = p0 + u * GPB < end;
#pragma unroll
        for (int g = 0; g < G; ++g) {
          float sdot = 0.f;
#pragma unroll
          for (int k = 0; k < N; ++k) sdot = fmaf(qr[g][k], kf[k], sdot);
          sdot = group_sum<GS>(sdot);
          sc[g][u] = ok ? sdot : kNegBig;
        }
      } else {
#pragma unroll
        for (int g = 0; g < G; ++g) sc[g][u] = kNegBig;
      }
    }
#pragma unroll
    for (int g = 0; g < G; ++g) {
      float mn = mx[g];
#pragma unroll
      for (int u = 0; u < U; ++u) mn = fmaxf(mn, sc[g][u]);
      const float corr = __expf(mx[g] - mn);
      mx[g] = mn;
      l[g] *= corr;
#pragma unroll
      for (int k = 0; k < N; ++k) acc[g][k] *= corr;
#pragma unroll
      for (int u = 0; u < U; ++u) sc[g][u] = p0 + u * GPB < end ? __expf(sc[g][u] - mn) : 0.f;
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (b0 + u * GPB < end) {
        float vf[N];
        Pack<WT>::unpack(vv[u], vf);
#pragma unroll
        for (int g = 0; g < G; ++g) {
          l[g] += sc[g][u];
#pragma unroll
          for (int k = 0; k < N; ++k) acc[g][k] = fmaf(sc[g][u], vf[k], acc[g][k]);
        }
      }
    }
  };
  // Two register sets alternate, so a block's loads stay in flight while the block before it is used
  // (copying one set into the other would wait for them).  The load behind the last block is clamped to
  // valid rows and never used.  The trip count is the same for every group of the workgroup.
  constexpr int STEP = U * GPB;
  const int nb = start < end ? (end - start + STEP - 1) / STEP : 0;
  int p0 = start + grp;
  if (nb > 0) load_block(p0, ku, vu);
  for (int i = 0; i + 2 <= nb; i += 2, p0 += 2 * STEP) {
    load_block(p0 + STEP, kn, vn);
    __builtin_amdgcn_sched_barrier(0);
    process(p0, ku, vu);
    load_block(p0 + 2 * STEP, ku, vu);
    __builtin_amdgcn_sched_barrier(0);
    process(p0 + STEP, kn, vn);
  }
  if (nb & 1) process(p0, ku, vu);

  // merge the groups of a wave through shuffles (same lane j of every group holds the same dims),
  // then the waves of the workgroup through LDS, both in fixed order
#pragma unroll
  for (int o = GS; o < kWave; o <<= 1) {
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const float m2 = __shfl_xor(mx[g], o, kWave);
      const float l2 = __shfl_xor(l[g], o, kWave);
      const float M = fmaxf(mx[g], m2);
      const float w1 = __expf(mx[g] - M), w2 = __expf(m2 - M);
      l[g] = l[g] * w1 + l2 * w2;
#pragma unroll
      for (int k = 0; k < N; ++k) {
        const float a2 = __shfl_xor(acc[g][k], o, kWave);
        acc[g][k] = acc[g][k] * w1 + a2 * w2;
      }
      mx[g] = M;
    }
  }
  constexpr int NW = BLOCK / kWave;
  const int wave = tid >> 6;
  if ((tid & 63) < GS) {                    // the wave's first group writes the wave's record
#pragma unroll
    for (int g = 0; g < G; ++g) {
      float *rec = merge + (wave * G + g) * REC;
      if (j == 0) { rec[0] = mx[g]; rec[1] = l[g]; }
#pragma unroll
      for (int k = 0; k < N; ++k) rec[2 + j * N + k] = acc[g][k];
    }
  }
  __syncthreads();
  for (int o = tid; o < G * HD; o += BLOCK) {
    const int g = o / HD, dim = o % HD;
    float M = kNegBig;
#pragma unroll
    for (int r = 0; r < NW; ++r) M = fmaxf(M, merge[(r * G + g) * REC]);
    float L = 0.f, A = 0.f;
#pragma unroll
    for (int r = 0; r < NW; ++r) {
      const float *rec = merge + (r * G + g) * REC;
      const float w = __expf(rec[0] - M);
      L = fmaf(rec[1], w, L);
      A = fmaf(rec[2 + dim], w, A);
    }
    const int head = kvh * G + g;
    if (n_splits == 1) {
      aout[head * HD + dim] = A / L;
    } else {
      float *pr = partials + ((size_t)head * n_splits + split) * REC;
      if (dim == 0) { st_agent(pr, M); st_agent(pr + 1, L); }
      st_agent(pr + 2 + dim, A);
    }
  }
  if (n_splits > 1) {
    // The last workgroup of this KV head to get here merges the splits.  The hand-over between
    // workgroups (other compute units, other L2 slices) uses no cache-wide fence: the partials are
    // written and read with agent-scope accesses, every wave waits for its own stores to complete,
    // and only then does the workgroup count itself in.  (A release fence per workgroup writes the
    // whole L2 back; measured, it costs more than the attention itself.)
    stores_done();
    __syncthreads();
    if (tid == 0) {
      const int prev = __hip_atomic_fetch_add(&counters[kvh * kCounterStride], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      *s_last = (prev == n_splits - 1);
    }
    __syncthreads();
    if (*s_last) {
      // Splits are added in index order.  Everything the merge needs is requested at once -- the (max, sum)
      // pair of every (head, split), one pair per thread, and this thread's accumulator element of up to
      // kMergeBatch splits -- so a merge of up to kMergeBatch splits waits for one trip past the L2, not
      // one per batch and output.  The pairs go through LDS (the group-merge records are dead by now):
      // lm/ll = max and sum per (head, split), lw = exp(max - head's max).
      constexpr int OPT = (G * HD + BLOCK - 1) / BLOCK;      // outputs per thread
      float *lm = merge, *ll = merge + G * kMaxAttnSplits, *lw = merge + 2 * G * kMaxAttnSplits;
      float pa[OPT][kMergeBatch];
      auto load_acc = [&](int s0) {
#pragma unroll
        for (int r = 0; r < OPT; ++r) {
          const int o = min(tid + r * BLOCK, G * HD - 1), g = o / HD, dim = o % HD;
          const float *pr = partials + (size_t)(kvh * G + g) * n_splits * REC + 2 + dim;
#pragma unroll
          for (int k = 0; k < kMergeBatch; ++k) pa[r][k] = ld_agent(pr + (size_t)min(s0 + k, n_splits - 1) * REC);
        }
      };
      float my_m = kNegBig, my_l = 0.f;
      static_assert(G * kMaxAttnSplits <= BLOCK, "one (max, sum) pair per thread");
      if (tid < G * n_splits) {
        const float *ps = partials + ((size_t)(kvh * G + tid / n_splits) * n_splits + tid % n_splits) * REC;
        my_m = ld_agent(ps); my_l = ld_agent(ps + 1);
      }
      load_acc(0);
      if (tid < G * n_splits) { lm[tid] = my_m; ll[tid] = my_l; }
      __syncthreads();
      if (tid < G * n_splits) {
        const int g = tid / n_splits;
        float M = kNegBig;
        for (int s2 = 0; s2 < n_splits; ++s2) M = fmaxf(M, lm[g * n_splits + s2]);
        lw[tid] = __expf(my_m - M);
      }
      __syncthreads();
      float A[OPT], L[OPT];
#pragma unroll
      for (int r = 0; r < OPT; ++r) { A[r] = 0.f; L[r] = 0.f; }
      for (int s0 = 0; s0 < n_splits; s0 += kMergeBatch) {
        if (s0 > 0) load_acc(s0);
#pragma unroll
        for (int r = 0; r < OPT; ++r) {
          const int g = min(tid + r * BLOCK, G * HD - 1) / HD;
#pragma unroll
          for (int k = 0; k < kMergeBatch; ++k) {
            if (s0 + k < n_splits) {
              const float w = lw[g * n_splits + s0 + k];
              L[r] = fmaf(ll[g * n_splits + s0 + k], w, L[r]);
              A[r] = fmaf(pa[r][k], w, A[r]);
            }
          }
        }
      }
#pragma unroll
      for (int r = 0; r < OPT; ++r) {
        const int o = tid + r * BLOCK;
        if (o < G * HD) aout[(kvh * G + o / HD) * HD + o % HD] = A[r] / L[r];
      }
      // ready for the next use (a later launch or a later phase)
      if (tid == 0) __hip_atomic_store(&counters[kvh * kCounterStride], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
  __syncthreads();   // merge / s_last may be reused by the caller
}

constexpr int kAttnLdsPages = 2048;   // page-table entries the attention kernel keeps in LDS

// grid = (n_kv, n_splits)
template <typename WT, int HD, int G>
__global__ __launch_bounds__(kGBlock) void k_attn(Common c, int role, int layer, const float *q, float *aout,
                                                  float *partials, int *counters) {
  // one record per wave and query head (the groups of a wave are merged through shuffles first); the merge of
  // the splits reuses it for 3 * G * kMaxAttnSplits floats
  __shared__ float merge[(kGBlock / kWave) * G * (HD + 2)];
  static_assert((kGBlock / kWave) * (HD + 2) >= 3 * kMaxAttnSplits, "the split merge's arrays fit the records");
  __shared__ int s_last;
  __shared__ int32_t s_ptab[kAttnLdsPages];
  // the page table does not depend on the state: copy it to LDS while the state is being read
  const bool lds_pt = c.dm.n_pages <= kAttnLdsPages;
  if (lds_pt)
    for (int i = threadIdx.x; i < c.dm.n_pages; i += kGBlock) s_ptab[i] = c.page_table[i];
  const StageIn si = stage_in(c, role);
  if (!si.active) return;
  __syncthreads();
  // two calls, not one with a selected pointer: a pointer that may be LDS or global memory makes every
  // page lookup a flat load, and waiting for a flat load waits for all K/V loads in flight as well
  if (lds_pt) attn_unit<WT, HD, G, kGBlock>(c, s_ptab, layer, si.pos, blockIdx.x, blockIdx.y, gridDim.y, q, aout, partials, counters, merge, &s_last);
  else attn_unit<WT, HD, G, kGBlock>(c, c.page_table, layer, si.pos, blockIdx.x, blockIdx.y, gridDim.y, q, aout, partials, counters, merge, &s_last);
}

// ------------------------------------------------------------------------------------------
// a5 / a7: out[r] = resid[r] + W[r,:] . vin   (o_proj and down_proj with the residual add fused).
// A task is ONE row (a trip = four column blocks of it): these matrices have few rows (d), and with
// two rows per wave only 8 waves per CU would be streaming; one row per wave gives 16 (measured on the
// 7B shapes: o_proj 10.3 -> 8.7 us, down 21.1 -> 18.7 us).  Per row the products are added in the same
// order as in the two-row form.  Dynamic LDS = C floats, padded to whole column blocks.
constexpr int kProjTripBlocks = 4;
template <typename WT, int DEPTH>
__global__ __launch_bounds__(kGBlock) void k_proj_resid(Common c, int role, const float *vin, int C,
                                                        const WT *W, int n_rows, int resid_sel, int out_sel) {
  extern __shared__ __align__(16) float xs[];
  CopyStage<kGBlock> in;
  in.issue(vin, C);                       // the input buffer's address never depends on the state
  const StageIn si = stage_in(c, role);
  if (!si.active) return;
  constexpr int KB = kProjTripBlocks;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int nwg = active_workgroups(c, role);
  if ((int)blockIdx.x >= nwg) return;
  const int gw = blockIdx.x * kGWaves + wave, tw = nwg * kGWaves;
  const WT *rows[1];
  auto set_rows = [&](int task) { rows[0] = W + (size_t)task * C; };
  Trips<WT, 1, KB, DEPTH> trips;
  trips.start(rows, gw, n_rows, tw, C, set_rows);
  in.template finish<WT>(C, xs);
  const float *resid = xslot(c, resid_sel);
  float *out = xslot(c, out_sel);
  trips.run(rows, gw, n_rows, tw, C, xs, set_rows, [&](int task, const float (&sum)[1]) {
    if (lane == 0) out[task] = resid[task] + sum[0];
  });
}

// The same projection for input vectors too long for three workgroups per compute unit to stage whole (more than
// 13312 floats: the down projection of the 13B and 8B shapes, 55-57 KB): the columns are walked in slabs of Cs
// (a multiple of a column block), one slab staged at a time, so a workgroup needs half the LDS and all of them are
// resident at once.  With the whole vector staged, 640 workgroups of 55 KB ran two per compute unit in 1.25
// rounds (13B: 29.2 us for 141.6 MB).  Every lane's FMA chain over its columns runs on from slab to slab (the
// running sums of up to kSlabRows rows per wave wait in LDS while the next slab is staged) and is reduced once at
// the end: per row the products are added in the single-slab order, the results are the same bit for bit.
// Dynamic LDS = Cs floats padded to whole column blocks.
constexpr int kSlabRows = 4;          // rows per wave whose running sums are kept across slabs; more rows: another round
constexpr int kSlabAbove = 13312;     // input lengths above this are walked in slabs
template <typename WT, int DEPTH>
__global__ __launch_bounds__(kGBlock) void k_proj_resid_slabs(Common c, int role, const float *vin, int C, int Cs,
                                                              const WT *W, int n_rows, int resid_sel, int out_sel) {
  extern __shared__ __align__(16) float xs[];
  __shared__ float carry[kSlabRows * kGBlock];
  CopyStage<kGBlock, kCopyPer / 2> in;    // a slab is at most half of the longest vector
  in.issue(vin, C < Cs ? C : Cs);         // the first slab; the input buffer's address never depends on the state
  const StageIn si = stage_in(c, role);
  if (!si.active) return;
  constexpr int KB = kProjTripBlocks;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int nwg = active_workgroups(c, role);
  if ((int)blockIdx.x >= nwg) return;
  const int tw = nwg * kGWaves;
  const float *resid = xslot(c, resid_sel);
  float *out = xslot(c, out_sel);
  // every wave of the workgroup goes through the same rounds and slabs (barriers); wave 0 has the most rows
  const int first = blockIdx.x * kGWaves;
  const int rows_wave0 = first < n_rows ? (n_rows - first + tw - 1) / tw : 0;
  const int rounds = (rows_wave0 + kSlabRows - 1) / kSlabRows;
  bool staged_first = false;
  for (int r = 0; r < rounds; ++r) {
    const int base = first + wave + r * kSlabRows * tw;            // this wave's first row of the round
    const int limit = min(n_rows, base + kSlabRows * tw);          // its rows: base, base + tw, ... below limit
    for (int c0 = 0; c0 < C; c0 += Cs) {
      const int w = C - c0 < Cs ? C - c0 : Cs;
      const WT *rows[1];
      auto set_rows = [&](int task) { rows[0] = W + (size_t)task * C + c0; };
      Trips<WT, 1, KB, DEPTH> trips;
      trips.start(rows, base, limit, tw, w, set_rows);             // weights do not wait for the staging
      if (staged_first) {
        __syncthreads();                                           // the slab before has been read by every wave
        in.issue(vin + c0, w);
      }
      in.template finish<WT>(w, xs);
      staged_first = true;
      int tb = 0, te = 0;                                          // index of the row inside the round
      const bool last = c0 + Cs >= C;
      trips.run_chained(rows, base, limit, tw, w, xs, set_rows,
                        [&](int) { const float v = c0 == 0 ? 0.f : carry[tb * kGBlock + threadIdx.x]; ++tb; return v; },
                        [&](int task, float sum) {
                          if (!last) {
                            carry[te * kGBlock + threadIdx.x] = sum;
                          } else {
                            const float s0 = wave_sum(sum);
                            if (lane == 0) out[task] = resid[task] + s0;
                          }
                          ++te;
                        });
    }
  }
}

// ------------------------------------------------------------------------------------------
// a2 + a6: RMSNorm + gate/up GEMV + SwiGLU: mout[i] = silu(Wg[i,:].xn) * (Wu[i,:].xn).
// A task is the pair (gate row i, up row i).
template <typename WT, int DEPTH>
__global__ __launch_bounds__(kGBlock) void k_gate_up(Common c, int role, int xin_sel, const float *gain,
                                                     const WT *wgu, float *mout) {
  extern __shared__ __align__(16) float xs[];
  __shared__ float red[kGWaves];
  const Dims &m = c.dm;
  const int d = m.d, f = m.f;
  NormStage<WT, kGBlock> in;
  const bool early = static_slot(xin_sel);
  if (early) in.issue(c.xbuf + (size_t)xin_sel * d, (const WT *)nullptr, gain, d);
  const StageIn si = stage_in(c, role);
  if (!si.active) return;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int nwg = active_workgroups(c, role);
  if ((int)blockIdx.x >= nwg) return;
  const int gw = blockIdx.x * kGWaves + wave, tw = nwg * kGWaves;
  const WT *rows[kTripRows];
  auto set_rows = [&](int task) {
    rows[0] = wgu + (size_t)task * d;
    rows[1] = wgu + (size_t)(f + task) * d;
  };
  Trips<WT, kTripRows, kTripBlocks, DEPTH> trips;
  if (!early) in.issue(xslot(c, xin_sel), (const WT *)nullptr, gain, d);
  trips.start(rows, gw, f, tw, d, set_rows);
  in.finish(d, m.eps, xs, red, nullptr);
  trips.run(rows, gw, f, tw, d, xs, set_rows, [&](int task, const float (&sum)[kTripRows]) {
    const float g = sum[0], u = sum[1];
    if (lane == 0) mout[task] = g / (1.0f + __expf(-g)) * u;
  });
}

// ------------------------------------------------------------------------------------------
// a8 / a9: head = RMSNorm + vocab projection + argmax (exit head and LM head share this kernel).
// A task is two consecutive vocabulary rows.  Each workgroup reduces its rows to one
// (value, index) candidate in cand[blockIdx.x]; the commit kernel finishes the reduction over
// gridDim.x candidates.  logits_log != nullptr additionally stores the logits (parity harness);
// logits_out != nullptr receives all V logits of this head (sampling needs the distribution).
template <typename WT, int DEPTH>
__global__ __launch_bounds__(kGBlock) void k_head(Common c, int role, int xin_sel, const float *gain,
                                                  const WT *W, float2 *cand, float *logits_log, int is_lm,
                                                  float *logits_out) {
  extern __shared__ __align__(16) float xs[];
  __shared__ float red[kGWaves];
  __shared__ float bv[kGWaves];
  __shared__ int bi[kGWaves];
  const Dims &m = c.dm;
  const int d = m.d, V = m.V;
  NormStage<WT, kGBlock> in;
  const bool early = static_slot(xin_sel);
  if (early) in.issue(c.xbuf + (size_t)xin_sel * d, (const WT *)nullptr, gain, d);
  const StageIn si = stage_in(c, role);
  if (!si.active) return;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int n_tasks = (V + 1) >> 1;
  const int nwg = active_workgroups(c, role);
  if ((int)blockIdx.x >= nwg) {     // the commit kernel reads one candidate per launched workgroup
    if (threadIdx.x == 0) cand[blockIdx.x] = make_float2(-INFINITY, __int_as_float(kNoIndex));
    return;
  }
  const int gw = blockIdx.x * kGWaves + wave, tw = nwg * kGWaves;
  const WT *rows[kTripRows];
  auto set_rows = [&](int task) {
    rows[0] = W + (size_t)(2 * task) * d;
    rows[1] = W + (size_t)min(2 * task + 1, V - 1) * d;
  };
  Trips<WT, kTripRows, kTripBlocks, DEPTH> trips;
  if (!early) in.issue(xslot(c, xin_sel), (const WT *)nullptr, gain, d);
  trips.start(rows, gw, n_tasks, tw, d, set_rows);
  in.finish(d, m.eps, xs, red, nullptr);
  // logits row for the parity harness: row index = number of tokens committed so far
  float *lrow = nullptr;
  if (logits_log && is_lm) {
    const int row = (role == kPrefill) ? 0 : c.st->gen_count;
    if (row < m.debug_rows) lrow = logits_log + (size_t)row * V;
  }
  float best = -INFINITY;
  int besti = kNoIndex;
  trips.run(rows, gw, n_tasks, tw, d, xs, set_rows, [&](int task, const float (&sum)[kTripRows]) {
    const float s0 = sum[0], s1 = sum[1];
    const int r = 2 * task;
    if (better(s0, r, best, besti)) { best = s0; besti = r; }
    if (r + 1 < V && better(s1, r + 1, best, besti)) { best = s1; besti = r + 1; }
    if (lrow && lane == 0) { lrow[r] = s0; if (r + 1 < V) lrow[r + 1] = s1; }
    if (logits_out && lane == 0) { logits_out[r] = s0; if (r + 1 < V) logits_out[r + 1] = s1; }
  });
  if (lane == 0) { bv[wave] = best; bi[wave] = besti; }
  __syncthreads();
  if (threadIdx.x == 0) {
#pragma unroll
    for (int w = 1; w < kGWaves; ++w)
      if (better(bv[w], bi[w], best, besti)) { best = bv[w]; besti = bi[w]; }
    cand[blockIdx.x] = make_float2(best, __int_as_float(besti));
  }
}

// ------------------------------------------------------------------------------------------
// a10: finish both argmax reductions, compare draft with the verifier's token, commit, roll back.
// One workgroup.  kind: 0 vanilla step, 1 PPSD step, 2 prefill position (no head), 3 last prefill
// position (LM head ran), 4 one tick of the full pipeline schedule.
template <int BLOCK>
__device__ __forceinline__ int reduce_candidates(const float2 *cand, int n, int vocab, float *sv, int *si_) {
  constexpr int NW = BLOCK / kWave;
  float best = -INFINITY;
  int besti = kNoIndex;
  for (int k = threadIdx.x; k < n; k += BLOCK) {
    const float2 cnd = cand[k];
    const int idx = __float_as_int(cnd.y);
    if (better(cnd.x, idx, best, besti)) { best = cnd.x; besti = idx; }
  }
  wave_argmax(best, besti);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) { sv[threadIdx.x >> 6] = best; si_[threadIdx.x >> 6] = besti; }
  __syncthreads();
  best = sv[0]; besti = si_[0];
#pragma unroll
  for (int w = 1; w < NW; ++w)
    if (better(sv[w], si_[w], best, besti)) { best = sv[w]; besti = si_[w]; }
  return argmax_token(besti, vocab);
}

// Called by all BLOCK threads of ONE workgroup.  sv / si_: BLOCK/64 entries of LDS each.
template <int BLOCK>
__device__ __forceinline__ void commit_step(const Common &c, int kind, const float2 *cand_lm, int n_cand_lm,
                                            const float2 *cand_exit, int n_cand_exit, int32_t *out_tokens,
                                            int32_t *drafts_log, float *sv, int *si_) {
  DevState *st = c.st;
  const int nb = n_cand_lm;
  if (kind == 2 || kind == 3) {   // prefill
    if (!(st->prefill_pos < st->prefill_len)) return;
    int tok = -1;
    if (kind == 3) tok = reduce_candidates<BLOCK>(cand_lm, nb, c.dm.V, sv, si_);
    if (threadIdx.x == 0) {
      st->prefill_pos += 1;
      if (kind == 3) {
        st->t = st->prefill_len;
        st->last_token = tok;
        st->full = 0;
        st->gen_count = 1;
        drafts_log[0] = -1;
        // full pipeline schedule: only stage 0 has work, the committed token at its position
        for (int k = 0; k < kMaxStages; ++k) { st->pl_valid[k] = 0; st->pl_pos[k] = 0; }
        st->pl_valid[0] = 1; st->pl_pos[0] = st->prefill_len; st->pl_tok0 = tok; st->pl_par = 0;
      }
    }
    return;
  }
  if (!(st->n_out < st->target)) return;
  if (kind == 4) {
    // One tick of the ceil(N/E)-stage schedule (Sec. 4.1-4.2, Alg. 1).  Stage 0 always ran and
    // drafted the token after its own; if the last stage ran, its LM head gives the model's token
    // for the position after the one it carried.  That token is emitted and compared with the one
    // stage 0 used at that position.  Equal: every token moves one stage on.  Different: all
    // tokens in flight came from a wrong draft; their KV rows are dropped by not advancing past
    // them (the restart rewrites those positions before anything reads them) and stage 0 restarts
    // from the verified token.
    const int S = c.dm.n_stages;
    const int ran_last = st->pl_valid[S - 1];
    const int d_next = reduce_candidates<BLOCK>(cand_exit, n_cand_exit, c.dm.V, sv, si_);
    int v = -1;
    if (ran_last) v = reduce_candidates<BLOCK>(cand_lm, nb, c.dm.V, sv, si_);
    if (threadIdx.x == 0) {
      int n_ran = 0;
      for (int k = 0; k < S; ++k) n_ran += st->pl_valid[k] ? 1 : 0;
      st->stats[8] += 1;
      st->stats[9] += n_ran;
      if (n_ran > 1) st->stats[4] += 1; else st->stats[5] += 1;
      const int pos0 = st->pl_pos[0];
      st->pl_tok_at[pos0 & (kTokRing - 1)] = st->pl_tok0;
      bool flush = false;
      if (ran_last) {
        const int p = st->pl_pos[S - 1] + 1;                  // the position v belongs to
        const int d = st->pl_tok_at[p & (kTokRing - 1)];      // stage 0 has used a draft there (S >= 2)
        out_tokens[st->n_out] = v;
        drafts_log[st->gen_count] = d;
        st->n_out += 1; st->gen_count += 1;
        st->stats[0] += 1; st->stats[1] += 1;
        st->t = p; st->last_token = v;
        if (v == d) {
          st->stats[2] += 1;
        } else {
          st->stats[3] += 1; st->stats[6] += 1;
          st->stats[10] += pos0 - p + 1;                      // the rejected draft and all after it
          flush = true;
        }
      }
      if (flush) {
        for (int k = 1; k < S; ++k) st->pl_valid[k] = 0;
        st->pl_pos[0] = st->t;
        st->pl_tok0 = v;
      } else {
        for (int k = S - 1; k > 0; --k) { st->pl_valid[k] = st->pl_valid[k - 1]; st->pl_pos[k] = st->pl_pos[k - 1]; }
        st->pl_pos[0] = pos0 + 1;
        st->pl_tok0 = d_next;
        st->pl_par ^= 1;                                      // what the stages wrote becomes readable
      }
    }
    return;
  }
  const int full = st->full;
  if (kind == 0) {   // vanilla: the LM head's token is the next token
    const int v = reduce_candidates<BLOCK>(cand_lm, nb, c.dm.V, sv, si_);
    if (threadIdx.x == 0) {
      out_tokens[st->n_out] = v;
      drafts_log[st->gen_count] = -1;
      st->n_out += 1; st->gen_count += 1; st->t += 1; st->last_token = v;
      st->stats[0] += 1;
    }
    return;
  }
  // PPSD step
  const int d_next = reduce_candidates<BLOCK>(cand_exit, n_cand_exit, c.dm.V, sv, si_);   // draft stage always ran
  int v = -1;
  if (full) v = reduce_candidates<BLOCK>(cand_lm, nb, c.dm.V, sv, si_);
  if (threadIdx.x == 0) {
    if (!full) {                 // pipeline refill: nothing to commit yet
      st->draft = d_next;
      st->full = 1;
      st->cur ^= 1;              // the draft stage wrote hExit[cur ^ 1]
      st->stats[5] += 1;
    } else {
      const int d = st->draft;
      out_tokens[st->n_out] = v;
      drafts_log[st->gen_count] = d;
      st->n_out += 1; st->gen_count += 1;
      st->stats[0] += 1; st->stats[1] += 1; st->stats[4] += 1;
      if (v == d) {              // accept: h_{t+1}^E and d_{t+2} from this step stay valid
        st->stats[2] += 1;
        st->draft = d_next;
        st->cur ^= 1;
      } else {                   // reject: drop the draft's KV row (layers 1..E) by not advancing
        st->stats[3] += 1;       // past it; the refill step rewrites position t+1
        st->stats[6] += 1;
        st->full = 0;
      }
      st->t += 1;
      st->last_token = v;
    }
  }
}

__global__ __launch_bounds__(kBlock) void k_commit(Common c, int kind, const float2 *cand_lm,
                                                   const float2 *cand_exit, int32_t *out_tokens,
                                                   int32_t *drafts_log) {
  __shared__ float sv[kWavesPerBlock];
  __shared__ int si_[kWavesPerBlock];
  commit_step<kBlock>(c, kind, cand_lm, c.dm.head_blocks, cand_exit, c.dm.head_blocks, out_tokens, drafts_log, sv, si_);
}

// ------------------------------------------------------------------------------------------
// Stochastic verification (Sec. 3.1, Eq. 1-2): sampled drafts, acceptance with probability
// min(1, q(d) / p(d)), a rejected draft replaced by a token from normalise(max(0, q - p)).
//
// Random numbers are a pure function of (seed, position, purpose): the splitmix64 output function
// on a key built from the three, reduced to a 24-bit fraction (exact in fp32), so the stream does
// not depend on the schedule.
constexpr int kSBlock = 1024;                        // threads of the sampling workgroup
constexpr int kSWaves = kSBlock / kWave;
enum Purpose : int { kPurDraft = 0, kPurAccept = 1, kPurResample = 2, kPurVanilla = 3 };

__device__ __forceinline__ float uniform24(uint32_t seed, int pos, int purpose) {
  unsigned long long z = (unsigned long long)seed ^ ((unsigned long long)pos * 0xD1342543DE82EF95ull) ^
                         ((unsigned long long)purpose * 0xA0761D6478BD642Full);
  z += 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  z ^= z >> 31;
  return (float)(uint32_t)(z >> 40) * (1.0f / 16777216.0f);
}

// Workgroup-wide helpers of the sampling kernel (kSBlock threads; buf: kSWaves floats of LDS).
__device__ __forceinline__ float sblock_max(float v, float *buf) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
  __syncthreads();
  if ((threadIdx.x & 63) == 0) buf[threadIdx.x >> 6] = v;
  __syncthreads();
  float m = buf[0];
  for (int w = 1; w < kSWaves; ++w) m = fmaxf(m, buf[w]);
  return m;
}

// Inverse-CDF sampling in index order over V non-negative weights wf(i): the first k with
// sum_{i<=k} w_i > u * sum_i w_i.  Thread j owns the contiguous chunk [j*per, (j+1)*per); sums run
// in index order inside a chunk and in thread order across chunks, and the threshold is taken
// against the very total those sums give, so the decision is a deterministic function of the weights.
// Returns the index in every thread; *total_out (if given) receives the total.  scan: kSBlock floats of LDS.
template <typename WF>
__device__ __forceinline__ int sample_index(WF &&wf, int V, float u, float *scan, int *s_pick, float *total_out) {
  const int per = (V + kSBlock - 1) / kSBlock;
  const int lo = threadIdx.x * per, hi = min(V, lo + per);
  float mine = 0.f;
  for (int i = lo; i < hi; ++i) mine += wf(i);
  __syncthreads();
  scan[threadIdx.x] = mine;
  __syncthreads();
  if (threadIdx.x == 0) {                       // exclusive scan in thread order (1024 adds: negligible)
    float run = 0.f;
    for (int j = 0; j < kSBlock; ++j) { const float v = scan[j]; scan[j] = run; run += v; }
    scan[kSBlock] = run;
    *s_pick = -1;
  }
  __syncthreads();
  const float total = scan[kSBlock];
  const float thr = u * total;
  const float before = scan[threadIdx.x];
  const float after = threadIdx.x + 1 < kSBlock ? scan[threadIdx.x + 1] : total;
  if (mine > 0.f && before <= thr && after > thr) {   // exactly one thread: the prefix sums are monotone
    float run = before;
    int k = -1;
    for (int i = lo; i < hi; ++i) {
      run += wf(i);
      if (run > thr) { k = i; break; }
    }
    if (k < 0) {                                 // rounding: the chunk's own sum fell short; its last positive weight
      for (int i = hi - 1; i >= lo; --i) if (wf(i) > 0.f) { k = i; break; }
    }
    *s_pick = k;
  }
  __syncthreads();
  int k = *s_pick;
  if (k < 0) {                                   // u * total rounded up to the total: the last positive weight
    if (threadIdx.x == 0) {
      int last = 0;
      for (int i = V - 1; i >= 0; --i) if (wf(i) > 0.f) { last = i; break; }
      *s_pick = last;
    }
    __syncthreads();
    k = *s_pick;
  }
  if (total_out) *total_out = total;
  __syncthreads();
  return k;
}

// One step's decision with sampling.  kind: 0 vanilla (token ~ q), 1 two-stage PPSD step,
// 3 last prefill position (token #0 ~ q), 4 one tick of the full pipeline schedule.  logits_lm /
// logits_exit: V floats each, written by the heads of this step.  probs: the distribution each
// in-flight draft was sampled from -- kind 1: [2][V], buffer st->cur & 1 belongs to the draft being
// verified, the other receives the new draft's; kind 4: [kMaxStages][V], indexed by position.
__global__ __launch_bounds__(kSBlock) void k_commit_sample(Common c, int kind, const float *logits_lm,
                                                           const float *logits_exit, float *probs, float inv_temp,
                                                           uint32_t seed, int32_t *out_tokens, int32_t *drafts_log) {
  __shared__ float scan[kSBlock + 1];
  __shared__ float buf[kSWaves];
  __shared__ int s_pick;
  DevState *st = c.st;
  const int V = c.dm.V;
  if (kind == 3) {
    if (!(st->prefill_pos < st->prefill_len)) return;
  } else if (!(st->n_out < st->target)) return;

  auto softmax_weights = [&](const float *lg, float &mx) {
    float m = -INFINITY;
    for (int i = threadIdx.x; i < V; i += kSBlock) m = fmaxf(m, lg[i]);
    mx = sblock_max(m, buf);
  };

  if (kind == 0 || kind == 3) {
    float mq;
    softmax_weights(logits_lm, mq);
    const int pos = kind == 3 ? st->prefill_len : st->t + 1;        // the position the token will occupy
    const int tok = sample_index([&](int i) { return __expf((logits_lm[i] - mq) * inv_temp); }, V,
                                 uniform24(seed, pos, kPurVanilla), scan, &s_pick, nullptr);
    if (threadIdx.x == 0) {
      if (kind == 3) {
        st->prefill_pos += 1;
        st->t = st->prefill_len; st->last_token = tok; st->full = 0; st->gen_count = 1;
        drafts_log[0] = -1;
        for (int k = 0; k < kMaxStages; ++k) { st->pl_valid[k] = 0; st->pl_pos[k] = 0; }
        st->pl_valid[0] = 1; st->pl_pos[0] = st->prefill_len; st->pl_tok0 = tok; st->pl_par = 0;
      } else {
        out_tokens[st->n_out] = tok;
        drafts_log[st->gen_count] = -1;
        st->n_out += 1; st->gen_count += 1; st->t += 1; st->last_token = tok;
        st->stats[0] += 1;
      }
    }
    return;
  }

  // ---- a PPSD step: two-stage (kind 1) or one tick of the full pipeline schedule (kind 4).
  // ran_verify: the last stage produced the full model's distribution for position pos, whose draft d
  // was sampled from p_cur; the first stage always ran and produced the distribution for position pos_d.
  const int S = c.dm.n_stages;
  int ran_verify, pos, pos_d, d;
  const float *p_cur;
  float *p_next;
  if (kind == 1) {
    const int cur = st->cur & 1;
    ran_verify = st->full;
    pos = st->t + 1;
    pos_d = (ran_verify ? st->t + 1 : st->t) + 1;
    d = st->draft;
    p_cur = probs + (size_t)cur * V;
    p_next = probs + (size_t)(cur ^ 1) * V;
  } else {
    const int pos0 = st->pl_pos[0];
    if (threadIdx.x == 0) st->pl_tok_at[pos0 & (kTokRing - 1)] = st->pl_tok0;   // the token stage 0 used this tick
    __syncthreads();
    ran_verify = st->pl_valid[S - 1];
    pos = st->pl_pos[S - 1] + 1;
    pos_d = pos0 + 1;
    d = st->pl_tok_at[pos & (kTokRing - 1)];
    p_cur = probs + (size_t)(pos & (kMaxStages - 1)) * V;        // kept since the tick that drafted position pos
    p_next = probs + (size_t)(pos_d & (kMaxStages - 1)) * V;
  }
  float mp;
  softmax_weights(logits_exit, mp);
  float sp;
  const int d_next = sample_index([&](int i) { return __expf((logits_exit[i] - mp) * inv_temp); }, V,
                                  uniform24(seed, pos_d, kPurDraft), scan, &s_pick, &sp);
  for (int i = threadIdx.x; i < V; i += kSBlock) p_next[i] = __expf((logits_exit[i] - mp) * inv_temp) / sp;

  int tok = -1, ok = 0;
  if (ran_verify) {
    float mq;
    softmax_weights(logits_lm, mq);
    // total of the target's weights, summed the way sample_index sums
    float sq;
    (void)sample_index([&](int i) { return __expf((logits_lm[i] - mq) * inv_temp); }, V, 0.f, scan, &s_pick, &sq);
    const float qd = __expf((logits_lm[d] - mq) * inv_temp) / sq;
    const float pd = p_cur[d];
    ok = uniform24(seed, pos, kPurAccept) * pd <= qd;
    if (ok) {
      tok = d;
    } else {
      auto resid = [&](int i) { return fmaxf(0.f, __expf((logits_lm[i] - mq) * inv_temp) / sq - p_cur[i]); };
      float sr;
      tok = sample_index(resid, V, uniform24(seed, pos, kPurResample), scan, &s_pick, &sr);
      if (!(sr > 0.f))                                               // q == p to rounding: take the token from q
        tok = sample_index([&](int i) { return __expf((logits_lm[i] - mq) * inv_temp); }, V,
                           uniform24(seed, pos, kPurResample), scan, &s_pick, nullptr);
    }
  }
  __syncthreads();
  if (threadIdx.x != 0) return;
  if (kind == 1) {
    if (!ran_verify) {
      st->draft = d_next; st->full = 1; st->cur ^= 1; st->stats[5] += 1;
    } else {
      out_tokens[st->n_out] = tok;
      drafts_log[st->gen_count] = d;
      st->n_out += 1; st->gen_count += 1;
      st->stats[0] += 1; st->stats[1] += 1; st->stats[4] += 1;
      if (ok) {
        st->stats[2] += 1; st->draft = d_next; st->cur ^= 1;
      } else {
        st->stats[3] += 1; st->stats[6] += 1; st->full = 0;
      }
      st->t += 1;
      st->last_token = tok;
    }
    return;
  }
  // kind 4: the tick's bookkeeping, as in the greedy commit
  int n_ran = 0;
  for (int k = 0; k < S; ++k) n_ran += st->pl_valid[k] ? 1 : 0;
  st->stats[8] += 1;
  st->stats[9] += n_ran;
  if (n_ran > 1) st->stats[4] += 1; else st->stats[5] += 1;
  const int pos0 = st->pl_pos[0];
  bool flush = false;
  if (ran_verify) {
    out_tokens[st->n_out] = tok;
    drafts_log[st->gen_count] = d;
    st->n_out += 1; st->gen_count += 1;
    st->stats[0] += 1; st->stats[1] += 1;
    st->t = pos; st->last_token = tok;
    if (ok) {
      st->stats[2] += 1;
    } else {
      st->stats[3] += 1; st->stats[6] += 1;
      st->stats[10] += pos0 - pos + 1;
      flush = true;
    }
  }
  if (flush) {
    for (int k = 1; k < S; ++k) st->pl_valid[k] = 0;
    st->pl_pos[0] = st->t;
    st->pl_tok0 = tok;
  } else {
    for (int k = S - 1; k > 0; --k) { st->pl_valid[k] = st->pl_valid[k - 1]; st->pl_pos[k] = st->pl_pos[k - 1]; }
    st->pl_pos[0] = pos0 + 1;
    st->pl_tok0 = d_next;
    st->pl_par ^= 1;
  }
}

// Host-requested state edits (tiny, one thread): new prefill / new decode target.
__global__ void k_begin_prefill(DevState *st, int n_prompt, int start_pos) {
  if (threadIdx.x == 0 && blockIdx.x == 0) {
    st->t = -1; st->last_token = -1; st->full = 0; st->draft = -1; st->cur = 0;
    st->n_out = 0; st->target = 0; st->gen_count = 0;
    st->prefill_pos = start_pos; st->prefill_len = n_prompt;
    for (int k = 0; k < 12; ++k) st->stats[k] = 0;
    for (int k = 0; k < kMaxStages; ++k) { st->pl_valid[k] = 0; st->pl_pos[k] = 0; }
    st->pl_tok0 = -1; st->pl_par = 0;
  }
}

__global__ void k_begin_decode(DevState *st, int n_tokens) {
  if (threadIdx.x == 0 && blockIdx.x == 0) { st->n_out = 0; st->target = n_tokens; }
}

// Fill of a few ints (arrival counters of a scratch region about to be used).
__global__ void k_fill_int(int *p, int n, int v) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

// Does nothing (measurement support: what a launch, and an event between two launches, cost).
__global__ void k_nop(int *p) { if (p == (int *)1) *p = 0; }

// Streaming-read probe: what a pure read reaches on this chip.  One workgroup of kGBlock threads per
// CU stays resident; each wave walks contiguous 8 KB chunks (eight non-temporal 16-byte loads per
// lane in flight), chunk index = wave + k * waves.  (Measured best of grid-stride, chunked and
// row-wise patterns: 7.0-7.2 TB/s.)
constexpr int kProbeLoads = 8;
__global__ __launch_bounds__(kGBlock) void k_read_probe(const uint4 *buf, size_t n_vec, uint32_t *sink) {
  const int lane = threadIdx.x & 63;
  const size_t gw = (size_t)blockIdx.x * kGWaves + (threadIdx.x >> 6);
  const size_t tw = (size_t)gridDim.x * kGWaves;
  const size_t chunk = (size_t)kProbeLoads * kWave;          // vectors per chunk
  const size_t n_chunks = n_vec / chunk;
  uint32_t acc = 0;
  for (size_t c = gw; c < n_chunks; c += tw) {
    uint4 v[kProbeLoads];
#pragma unroll
    for (int j = 0; j < kProbeLoads; ++j) v[j] = ld16_stream(buf + c * chunk + j * kWave + lane);
#pragma unroll
    for (int j = 0; j < kProbeLoads; ++j) acc += v[j].x ^ v[j].y ^ v[j].z ^ v[j].w;
  }
  for (size_t i = n_chunks * chunk + gw * kWave + lane; i < n_vec; i += tw * kWave) {   // the tail
    const uint4 a = ld16_stream(buf + i);
    acc += a.x ^ a.y ^ a.z ^ a.w;
  }
  if (acc == 0x9e3779b9u) sink[0] = acc;   // practically never; keeps the loads alive
}

}  // namespace ppsd
