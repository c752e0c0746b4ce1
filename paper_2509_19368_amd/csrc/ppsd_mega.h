// Persistent-kernel engine: a whole ppsd_decode (or prefill) call in ONE cooperative launch.
//
// One workgroup of 512 threads per CU stays resident and walks the step's operations ("phases":
// QKV, attention, o_proj, gate/up, down of every layer, then the head) separated by grid
// barriers.  The draft stage and the verify stage of a PPSD step are zipped: phase k runs
// operation k of BOTH stages, so the two stages advance concurrently on disjoint waves
// (verify-while-draft, Sec. 4.2) and a step needs max(ops_draft, ops_verify) barriers instead of
// their sum.
//
// Weight streaming is software-pipelined across barriers: which weight bytes a wave reads next
// depends only on the static schedule, never on activations, so every wave issues the loads of
// its NEXT task (16 x 16 bytes per lane, possibly belonging to a later phase) before it finishes
// the current one and before it waits at a barrier.  HBM therefore keeps streaming while
// barriers, RMSNorm prologues and the (latency-bound) attention phase run.
//
// Every wait is bounded: a barrier that does not complete within kSpinLimit polls raises the
// abort flag, and every workgroup leaves the kernel at its next wait.
#pragma once

#include "ppsd_kernels.h"

namespace ppsd {

constexpr int kMBlock = 512;
constexpr int kMWaves = kMBlock / kWave;
constexpr int kTaskBlocks = 8;            // 16-byte column blocks per row per task
constexpr unsigned kSpinLimit = 1u << 20; // polls (each >= 1 us) before a barrier wait gives up

enum SegKind : int { SK_QKV = 0, SK_ATTN = 1, SK_OPROJ = 2, SK_GATEUP = 3, SK_DOWN = 4, SK_HEAD = 5 };

struct LayerPtrs {
  const float *attn_norm;
  const void *wqkv;
  const void *wo;
  const float *mlp_norm;
  const void *wgu;
  const void *wdown;
};

struct StageDesc {
  int32_t role;        // Role
  int32_t lo, hi;      // layers [lo, hi)
  int32_t slot;        // scratch set (q / a / m / partials / counters)
  int32_t xin_first;   // residual slot the first layer reads (and, with from_embed, receives the embedding)
  int32_t from_embed;
  int32_t xwork;       // residual slot used inside the stage
  int32_t xout_last;   // slot the last layer's down-projection writes
  int32_t head;        // 0 none, 1 LM head, 2 exit head, 3 LM head at the last prefill position only
  int32_t head_xin;
};

struct MegaArgs {
  Common cm;
  const LayerPtrs *layers;
  const void *embed;
  const float *final_norm;
  const void *lm_head;
  const float *exit_norm;
  const void *exit_head;
  float *q[2];
  float *a[2];
  float *m[2];
  float *partials[2];
  int *counters[2];
  float2 *cand_lm;
  float2 *cand_exit;
  float *logits;
  int32_t *out_tokens;
  int32_t *drafts;
  unsigned *bar;       // monotonic arrival counter, zeroed by the host before the launch
  int *abort_flag;     // zeroed by the host; nonzero after a barrier timeout
  StageDesc st[2];
  int32_t n_stages;
  int32_t zip;         // 1: stages share phases; 0: stage 0's phases, then stage 1's
  int32_t commit_kind; // 0 vanilla, 1 PPSD, 2 prefill
  int32_t max_steps;
  int32_t attn_splits;
  int32_t xs_stride;   // floats per staged-input region in LDS
  unsigned long long *trace;  // optional timeline of workgroup 0 (nullptr = off): 4 timestamps per phase
  int32_t trace_step;         // the step whose phases are recorded
  int32_t trace_wg;           // the workgroup that records
};

constexpr int kTraceSlots = 4;     // per phase: barrier passed, inputs staged, own tasks done, arrived
constexpr int kTracePhases = 512;

struct StageRun { int active, pos, tok, head_on; };

struct SegInfo {
  int kind, layer, units, C;   // units: stream units (row pairs); 0 for attention / inactive
  int active;
};

// ---------------------------------------------------------------- grid barrier (bounded)
__device__ __forceinline__ void grid_arrive(unsigned *bar) {
  __hip_atomic_fetch_add(bar, 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ bool grid_wait(unsigned *bar, unsigned target, int *abort_flag) {
  unsigned spins = 0;
  for (;;) {
    const unsigned v = __hip_atomic_load(bar, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (v >= target) break;
    ++spins;
    if ((spins & 31u) == 0) {
      if (__hip_atomic_load(abort_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) return false;
      if (spins > kSpinLimit) {
        __hip_atomic_store(abort_flag, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return false;
      }
    }
    __builtin_amdgcn_s_sleep(2);
  }
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
  return true;
}

// ---------------------------------------------------------------- static schedule helpers
__device__ __forceinline__ int stage_nops(const StageDesc &s) { return 5 * (s.hi - s.lo) + (s.head ? 1 : 0); }

__device__ __forceinline__ int n_phases(const MegaArgs &A) {
  const int n0 = stage_nops(A.st[0]);
  const int n1 = A.n_stages > 1 ? stage_nops(A.st[1]) : 0;
  return A.zip ? max(n0, n1) : n0 + n1;
}

// Operation `op` of stage `si` under this step's run state.
__device__ __forceinline__ SegInfo seg_info(const MegaArgs &A, int si, int op, const StageRun &run) {
  const StageDesc &s = A.st[si];
  const Dims &m = A.cm.dm;
  SegInfo g;
  g.active = 0; g.units = 0; g.C = 0; g.layer = 0; g.kind = SK_ATTN;
  if (op < 0 || op >= stage_nops(s) || !run.active) return g;
  const int nl = s.hi - s.lo;
  if (op < 5 * nl) {
    g.layer = s.lo + op / 5;
    g.kind = op % 5;
    g.active = 1;
    switch (g.kind) {
      case SK_QKV: g.units = (m.n_h + 2 * m.n_kv) * (m.hd >> 1); g.C = m.d; break;
      case SK_ATTN: g.units = 0; break;
      case SK_OPROJ: g.units = (m.d + 1) >> 1; g.C = m.n_h * m.hd; break;
      case SK_GATEUP: g.units = m.f; g.C = m.d; break;
      default: g.units = (m.d + 1) >> 1; g.C = m.f; break;   // SK_DOWN
    }
  } else {
    g.kind = SK_HEAD;
    g.active = run.head_on;
    g.units = g.active ? (m.V + 1) >> 1 : 0;
    g.C = m.d;
  }
  return g;
}

// The (up to two) segments of phase p: out[k] belongs to stage sidx[k].
struct PhaseSegs {
  SegInfo g0, g1;   // g0 belongs to stage s0, g1 to stage s1
  int s0, s1;
};

__device__ __forceinline__ PhaseSegs phase_segs(const MegaArgs &A, int p, const StageRun &run0, const StageRun &run1) {
  PhaseSegs ps;
  ps.s0 = 0; ps.s1 = 1;
  if (A.zip || A.n_stages == 1) {
    ps.g0 = seg_info(A, 0, p, run0);
    if (A.n_stages > 1) ps.g1 = seg_info(A, 1, p, run1);
    else { ps.g1 = ps.g0; ps.g1.active = 0; ps.g1.units = 0; }
  } else {
    const int n0 = stage_nops(A.st[0]);
    if (p < n0) { ps.g0 = seg_info(A, 0, p, run0); }
    else { ps.g0 = seg_info(A, 1, p - n0, run1); ps.s0 = 1; }
    ps.g1 = ps.g0; ps.g1.active = 0; ps.g1.units = 0;
  }
  return ps;
}

template <typename WT>
struct Task {
  int valid = 0;
  int p = 0;    // phase
  int u = 0;    // unit index within the phase's concatenated unit list
  int k = 0;    // which segment of the phase (0/1)
  int si = 0;   // stage index
  int kind = 0, layer = 0, ul = 0, ch = 0, nch = 1, C = 0;
  int nblk = 0;     // 16-byte column blocks in a row (the last one may be ragged)
  const WT *r0 = nullptr, *r1 = nullptr;
};

template <typename WT>
__device__ __forceinline__ void fill_task(const MegaArgs &A, Task<WT> &t, const SegInfo &g) {
  const Dims &m = A.cm.dm;
  constexpr int kStride = kWave * Pack<WT>::N;
  const LayerPtrs *lpp = A.layers + g.layer;
  LayerPtrs lp;
  lp.wqkv = uniform_ptr(lpp->wqkv); lp.wo = uniform_ptr(lpp->wo);
  lp.wgu = uniform_ptr(lpp->wgu); lp.wdown = uniform_ptr(lpp->wdown);
  t.kind = g.kind; t.layer = g.layer; t.C = g.C;
  const int nblk = (g.C + kStride - 1) / kStride;
  t.nblk = nblk;
  t.nch = (nblk + kTaskBlocks - 1) / kTaskBlocks;
  t.ch = 0;
  const int ul = t.ul;
  switch (g.kind) {
    case SK_QKV: {
      const int half = m.hd >> 1;
      const int head = ul / half, i = ul - head * half;
      t.r0 = (const WT *)lp.wqkv + (size_t)(head * m.hd + i) * m.d;
      t.r1 = t.r0 + (size_t)half * m.d;
    } break;
    case SK_GATEUP:
      t.r0 = (const WT *)lp.wgu + (size_t)ul * m.d;
      t.r1 = (const WT *)lp.wgu + (size_t)(m.f + ul) * m.d;
      break;
    case SK_OPROJ:
    case SK_DOWN: {
      const WT *W = (const WT *)(g.kind == SK_OPROJ ? lp.wo : lp.wdown);
      t.r0 = W + (size_t)(2 * ul) * g.C;
      t.r1 = W + (size_t)min(2 * ul + 1, m.d - 1) * g.C;
    } break;
    default: {   // SK_HEAD
      const StageDesc &s = A.st[t.si];
      const WT *W = (const WT *)(s.head == 2 ? A.exit_head : A.lm_head);
      t.r0 = W + (size_t)(2 * ul) * m.d;
      t.r1 = W + (size_t)min(2 * ul + 1, m.V - 1) * m.d;
    } break;
  }
}

// First task at or after (p, u) for a wave whose units are u, u + TW, ... in every phase.
template <typename WT>
__device__ __forceinline__ void find_task(const MegaArgs &A, const StageRun &run0, const StageRun &run1, int p, int u,
                                          int gw, int nph, Task<WT> &t) {
  t.valid = 0;
  while (p < nph) {
    const PhaseSegs ps = phase_segs(A, p, run0, run1);
    const int u0 = ps.g0.units, u1 = ps.g1.units;
    if (u < u0 + u1) {
      t.valid = 1; t.p = p; t.u = u;
      if (u < u0) { t.k = 0; t.ul = u; t.si = ps.s0; fill_task<WT>(A, t, ps.g0); }
      else { t.k = 1; t.ul = u - u0; t.si = ps.s1; fill_task<WT>(A, t, ps.g1); }
      break;
    }
    ++p;
    u = gw;
  }
  // everything about a task is wave-uniform: keep it in scalar registers
  t.valid = uniform(t.valid); t.p = uniform(t.p); t.u = uniform(t.u); t.k = uniform(t.k); t.si = uniform(t.si);
  t.kind = uniform(t.kind); t.layer = uniform(t.layer); t.ul = uniform(t.ul); t.ch = uniform(t.ch);
  t.nch = uniform(t.nch); t.C = uniform(t.C); t.nblk = uniform(t.nblk);
  t.r0 = uniform_ptr(t.r0); t.r1 = uniform_ptr(t.r1);
}

template <typename WT>
__device__ __forceinline__ void next_task(const MegaArgs &A, const StageRun &run0, const StageRun &run1,
                                          const Task<WT> &cur, int gw, int tw, int nph, Task<WT> &nx) {
  if (cur.ch + 1 < cur.nch) {
    nx = cur;
    nx.ch = cur.ch + 1;
    return;
  }
  find_task<WT>(A, run0, run1, cur.p, cur.u + tw, gw, nph, nx);
}

// Issues the task's loads.  Whole blocks are selected by wave-uniform branches; inside the ragged
// last block of a row the lanes past the end re-read the row's last 16 bytes (their products are
// skipped in accumulate), so no load is predicated per lane.  Every element of buf is (re)defined,
// which ends the live range of the buffer's previous contents.
template <typename WT>
__device__ __forceinline__ void prefetch(uint4 (&buf)[2 * kTaskBlocks], const Task<WT> &t) {
  constexpr int N = Pack<WT>::N;
  constexpr int kStride = kWave * N;
  const int lane = threadIdx.x & 63;
  const int b0 = t.ch * kTaskBlocks;
  const int nb = min(kTaskBlocks, t.nblk - b0);          // uniform
  const int last = t.C - N;
#pragma unroll
  for (int b = 0; b < kTaskBlocks; ++b) {
    if (b < nb) {
      const int c = min((b0 + b) * kStride + lane * N, last);
      const uint32_t off = (uint32_t)c * (uint32_t)sizeof(WT);
      buf[2 * b] = ld16_stream_global(t.r0, off);
      buf[2 * b + 1] = ld16_stream_global(t.r1, off);
    } else {
      buf[2 * b] = make_uint4(0u, 0u, 0u, 0u);
      buf[2 * b + 1] = make_uint4(0u, 0u, 0u, 0u);
    }
  }
}

template <typename WT>
__device__ __forceinline__ void clear_buf(uint4 (&buf)[2 * kTaskBlocks]) {
#pragma unroll
  for (int b = 0; b < 2 * kTaskBlocks; ++b) buf[b] = make_uint4(0u, 0u, 0u, 0u);
}

template <typename WT>
__device__ __forceinline__ void accumulate(const uint4 (&buf)[2 * kTaskBlocks], const Task<WT> &t, const float *xs,
                                           float &acc0, float &acc1) {
  constexpr int N = Pack<WT>::N;
  constexpr int kStride = kWave * N;
  const int lane = threadIdx.x & 63;
  const int c0 = t.ch * kTaskBlocks * kStride + lane * N;
#pragma unroll
  for (int b = 0; b < kTaskBlocks; ++b) {
    const int c = c0 + b * kStride;
    if (c < t.C) {
      float x[N], w0[N], w1[N];
#pragma unroll
      for (int k = 0; k < N; ++k) x[k] = xs[c + k];
      Pack<WT>::unpack(buf[2 * b], w0);
      Pack<WT>::unpack(buf[2 * b + 1], w1);
#pragma unroll
      for (int k = 0; k < N; ++k) acc0 = fmaf(w0[k], x[k], acc0);
#pragma unroll
      for (int k = 0; k < N; ++k) acc1 = fmaf(w1[k], x[k], acc1);
    }
  }
}

// Sum over a 512-thread workgroup; every thread gets the result.
__device__ __forceinline__ float mblock_sum(float v, float *red) {
  v = wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  float s = 0.f;
#pragma unroll
  for (int w = 0; w < kMWaves; ++w) s += red[w];
  return s;
}

// ------------------------------------------------------------------------------------------
template <typename WT, int HD, int G>
__global__ __launch_bounds__(kMBlock) void k_mega(MegaArgs A) {
  extern __shared__ float lds[];            // 2 staged-input regions; reused as the attention merge buffer
  __shared__ float red[kMWaves];
  __shared__ float bv[2][kMWaves];
  __shared__ int bi[2][kMWaves];
  __shared__ int s_flag;
  __shared__ int s_last;

  const Common &c = A.cm;
  const Dims &m = c.dm;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wg = blockIdx.x, nwg = gridDim.x;
  const int gw = wg * kMWaves + wave, tw = nwg * kMWaves;
  const int nph = n_phases(A);
  unsigned nbar = 0;                        // barriers this workgroup has arrived at

  for (int step = 0; step < A.max_steps; ++step) {
    // ---- the state is stable here: every workgroup is past the barrier that follows the commit
    volatile const DevState *vs = c.st;
    StageRun run0, run1;
    int cur_h;
    {
      const int t = uniform(vs->t), last = uniform(vs->last_token), full = uniform(vs->full), draft = uniform(vs->draft);
      const int running = uniform(vs->n_out) < uniform(vs->target);
      const int ppos = uniform(vs->prefill_pos), plen = uniform(vs->prefill_len);
      cur_h = uniform(vs->cur) & 1;
      auto resolve = [&](int s) {
        StageRun r;
        r.active = 0; r.pos = 0; r.tok = 0; r.head_on = 0;
        if (s >= A.n_stages) return r;
        const int role = A.st[s].role, head = A.st[s].head;
        if (role == kPrefill) {
          r.active = ppos < plen; r.pos = ppos;
          r.tok = r.active ? uniform(c.prompt[ppos]) : 0;
          r.head_on = r.active && (head == 1 || (head == 3 && ppos == plen - 1));
        } else if (role == kVanilla) {
          r.active = running; r.pos = t; r.tok = last; r.head_on = running && head != 0;
        } else if (role == kDraft) {
          r.active = running; r.pos = full ? t + 1 : t; r.tok = full ? draft : last;
          r.head_on = running && head != 0;
        } else {
          r.active = running && full; r.pos = t; r.tok = -1;
          r.head_on = r.active && head != 0;
        }
        return r;
      };
      run0 = resolve(0);
      run1 = resolve(1);
    }
    if (!run0.active && !run1.active) break;
    const int last_prefill = (A.commit_kind == 2) && (uniform(vs->prefill_pos) == uniform(vs->prefill_len) - 1);

    auto slot_ptr = [&](int sel) -> float * {
      int slot = sel;
      if (sel == kHExitCur) slot = 2 + cur_h;
      else if (sel == kHExitNext) slot = 2 + (cur_h ^ 1);
      return c.xbuf + (size_t)slot * m.d;
    };

    const bool tracing = A.trace != nullptr && step == A.trace_step && wg == A.trace_wg && nph <= kTracePhases;
    float bestv0 = -INFINITY, bestv1 = -INFINITY;     // running argmax of head segment 0 / 1 (wave-uniform)
    int besti0 = 0x7fffffff, besti1 = 0x7fffffff;
    int entered = -1;
    bool ok = true;

    // ---- leave-side work of one segment: publish this wave's head candidate
    auto seg_leave_publish = [&](int k, const SegInfo &g, float bvv, int bii) {
      if (g.active && g.kind == SK_HEAD && lane == 0) { bv[k][wave] = bvv; bi[k][wave] = bii; }
    };
    auto seg_leave_reduce = [&](int k, const SegInfo &g, int si) {   // thread 0 only
      if (g.active && g.kind == SK_HEAD) {
        float b = bv[k][0]; int bidx = bi[k][0];
        for (int w = 1; w < kMWaves; ++w)
          if (better(bv[k][w], bi[k][w], b, bidx)) { b = bv[k][w]; bidx = bi[k][w]; }
        float2 *cand = A.st[si].head == 2 ? A.cand_exit : A.cand_lm;
        cand[wg] = make_float2(b, __int_as_float(bidx));
      }
    };
    // ---- enter-side work of one segment: stage its input vector in LDS region k
    auto seg_stage = [&](int k, const SegInfo &g, int si, const StageRun &run) {
      if (!g.active) return;
      const StageDesc &s = A.st[si];
      const LayerPtrs *lpp = A.layers + g.layer;
      float *xs = lds + (size_t)k * A.xs_stride;
      const bool first_layer = g.layer == s.lo;
      if (g.kind == SK_QKV || g.kind == SK_GATEUP || g.kind == SK_HEAD) {
        const float *gain;
        const float *xf = nullptr;
        const WT *xrow = nullptr;
        float *copy_out = nullptr;
        if (g.kind == SK_QKV) {
          gain = uniform_ptr(lpp->attn_norm);
          if (first_layer && s.from_embed) {
            xrow = (const WT *)A.embed + (size_t)run.tok * m.d;
            if (wg == 0) copy_out = slot_ptr(s.xin_first);
          } else {
            xf = slot_ptr(first_layer ? s.xin_first : s.xwork);
          }
        } else if (g.kind == SK_GATEUP) {
          gain = uniform_ptr(lpp->mlp_norm);
          xf = slot_ptr(s.xwork);
        } else {
          gain = s.head == 2 ? A.exit_norm : A.final_norm;
          xf = slot_ptr(s.head_xin);
        }
        NormStage<WT, kMBlock> in;       // same code, same reduction order as the per-operation kernels
        in.issue(xf, xrow, gain, m.d);
        in.finish(m.d, m.eps, xs, red, copy_out);
      } else if (g.kind == SK_OPROJ || g.kind == SK_DOWN) {
        CopyStage<kMBlock> in;
        in.issue(g.kind == SK_OPROJ ? A.a[s.slot] : A.m[s.slot], g.C);
        in.finish(g.C, xs);
      }
    };
    // ---- attention is workgroup-level work done at phase entry (such a phase has no weight tasks)
    auto seg_attention = [&](int k, const SegInfo &g, int si, const StageRun &run) {
      if (!g.active || g.kind != SK_ATTN) return;
      const StageDesc &s = A.st[si];
      const int per = m.n_kv * A.attn_splits;
      // the two stages' units start half a grid apart so that they land on different workgroups
      const int first = (k == 0) ? wg : (wg + nwg / 2) % nwg;
      for (int u = first; u < per; u += nwg) {
        const int kvh = u / A.attn_splits, split = u - kvh * A.attn_splits;
        attn_unit<WT, HD, G, kMBlock>(c, c.page_table, g.layer, run.pos, kvh, split, A.attn_splits, A.q[s.slot], A.a[s.slot],
                                      A.partials[s.slot], A.counters[s.slot], lds, &s_last);
      }
    };

    // Leaves phases up to target-1 and enters phases up to target, in order, with all collective work.
    auto sync_to_phase = [&](int target) {
      while (entered < target && ok) {
        if (entered >= 0) {
          const PhaseSegs ps = phase_segs(A, entered, run0, run1);
          if (ps.g0.active || ps.g1.active) {
            // ---- leave: publish head candidates, then arrive
            seg_leave_publish(0, ps.g0, bestv0, besti0);
            seg_leave_publish(1, ps.g1, bestv1, besti1);
            __syncthreads();
            if (tracing && tid == 0) A.trace[entered * kTraceSlots + 2] = wall_clock64();
            if (tid == 0) {
              seg_leave_reduce(0, ps.g0, ps.s0);
              seg_leave_reduce(1, ps.g1, ps.s1);
              grid_arrive(A.bar);
              if (tracing) A.trace[entered * kTraceSlots + 3] = wall_clock64();
            }
            nbar += 1;
            bestv0 = -INFINITY; bestv1 = -INFINITY; besti0 = 0x7fffffff; besti1 = 0x7fffffff;
          }
        }
        ++entered;
        if (entered >= nph) break;
        const PhaseSegs ps = phase_segs(A, entered, run0, run1);
        if (!(ps.g0.active || ps.g1.active)) continue;
        // ---- enter: wait for every workgroup to have left the previous active phase
        if (nbar > 0) {
          if (tid == 0) s_flag = grid_wait(A.bar, nbar * (unsigned)nwg, A.abort_flag) ? 1 : 0;
          __syncthreads();
          if (!s_flag) { ok = false; break; }
        }
        if (tracing && tid == 0) A.trace[entered * kTraceSlots + 0] = wall_clock64();
        seg_stage(0, ps.g0, ps.s0, ps.s0 ? run1 : run0);
        seg_stage(1, ps.g1, ps.s1, run1);
        __syncthreads();
        if (tracing && tid == 0) A.trace[entered * kTraceSlots + 1] = wall_clock64();
        seg_attention(0, ps.g0, ps.s0, ps.s0 ? run1 : run0);
        seg_attention(1, ps.g1, ps.s1, run1);
      }
    };

    // ---- the step's weight tasks, double-buffered in registers
    uint4 bufA[2 * kTaskBlocks], bufB[2 * kTaskBlocks];
    float acc0 = 0.f, acc1 = 0.f;
    Task<WT> cur, nx;
    find_task<WT>(A, run0, run1, 0, gw, gw, nph, cur);
    if (cur.valid) prefetch<WT>(bufA, cur); else clear_buf<WT>(bufA);
    clear_buf<WT>(bufB);

    auto finish = [&](const Task<WT> &t) {   // epilogue of a unit: wave-reduce and write
      const float s0 = wave_sum(acc0), s1 = wave_sum(acc1);
      acc0 = 0.f; acc1 = 0.f;
      const StageDesc &s = A.st[t.si];
      const int pos = t.si ? run1.pos : run0.pos;
      switch (t.kind) {
        case SK_QKV: {
          if (lane == 0) {
            const int half = m.hd >> 1;
            const int h = t.ul / half, i = t.ul - h * half;
            float lo = s0, hi = s1;
            if (h < m.n_h + m.n_kv) {
              const float cs = c.rope_cos[(size_t)pos * half + i];
              const float sn = c.rope_sin[(size_t)pos * half + i];
              const float rlo = lo * cs - hi * sn;
              const float rhi = hi * cs + lo * sn;
              lo = rlo; hi = rhi;
            }
            if (h < m.n_h) {
              A.q[s.slot][h * m.hd + i] = lo;
              A.q[s.slot][h * m.hd + i + half] = hi;
            } else {
              const int which = (h < m.n_h + m.n_kv) ? 0 : 1;
              const int kvh = which ? h - m.n_h - m.n_kv : h - m.n_h;
              WT *dst = kv_row<WT>(c, c.page_table, t.layer, pos, kvh, which);
              dst[i] = Pack<WT>::from_float(lo);
              dst[i + half] = Pack<WT>::from_float(hi);
            }
          }
        } break;
        case SK_GATEUP:
          if (lane == 0) A.m[s.slot][t.ul] = s0 / (1.0f + __expf(-s0)) * s1;
          break;
        case SK_OPROJ:
        case SK_DOWN: {
          if (lane < 2 && 2 * t.ul + lane < m.d) {
            const bool first_layer = t.layer == s.lo, last_layer = t.layer == s.hi - 1;
            const float *resid = slot_ptr(t.kind == SK_OPROJ ? (first_layer ? s.xin_first : s.xwork) : s.xwork);
            float *out = slot_ptr(t.kind == SK_OPROJ ? s.xwork : (last_layer ? s.xout_last : s.xwork));
            const int r = 2 * t.ul + lane;
            out[r] = resid[r] + (lane == 0 ? s0 : s1);
          }
        } break;
        default: {   // SK_HEAD
          const int r = 2 * t.ul;
          float *lrow = nullptr;
          if (A.logits && s.head != 2) {
            const int row = (s.role == kPrefill) ? 0 : uniform(vs->gen_count);
            if (row < m.debug_rows) lrow = A.logits + (size_t)row * m.V;
          }
          float bvv = t.k ? bestv1 : bestv0;
          int bii = t.k ? besti1 : besti0;
          if (better(s0, r, bvv, bii)) { bvv = s0; bii = r; }
          if (r + 1 < m.V && better(s1, r + 1, bvv, bii)) { bvv = s1; bii = r + 1; }
          if (t.k) { bestv1 = bvv; besti1 = bii; } else { bestv0 = bvv; besti0 = bii; }
          if (lrow && lane == 0) { lrow[r] = s0; if (r + 1 < m.V) lrow[r + 1] = s1; }
        } break;
      }
    };

    // One transition site.  The current task's loads were issued an iteration earlier, so they are in
    // flight while the transition (barrier, input staging, attention) runs; the next task's loads are
    // issued right after it, before the current buffer is consumed.  The buffer roles alternate by a
    // wave-uniform parity.  After the last task the same site runs the remaining phase transitions.
    int parity = 0;
    for (;;) {
      sync_to_phase(cur.valid ? cur.p : nph);
      if (!ok || !cur.valid) break;
      next_task<WT>(A, run0, run1, cur, gw, tw, nph, nx);
      if (parity) { if (nx.valid) prefetch<WT>(bufA, nx); else clear_buf<WT>(bufA); }
      else { if (nx.valid) prefetch<WT>(bufB, nx); else clear_buf<WT>(bufB); }
      const float *xs = lds + (size_t)cur.k * A.xs_stride;
      if (parity) accumulate<WT>(bufB, cur, xs, acc0, acc1);
      else accumulate<WT>(bufA, cur, xs, acc0, acc1);
      if (cur.ch == cur.nch - 1) finish(cur);
      cur = nx;
      parity ^= 1;
    }
    if (!ok) return;

    // ---- commit: everyone waits for the last phase, workgroup 0 commits, everyone waits for that
    if (tid == 0) s_flag = grid_wait(A.bar, nbar * (unsigned)nwg, A.abort_flag) ? 1 : 0;
    __syncthreads();
    if (!s_flag) return;
    if (wg == 0) {
      const int kind = A.commit_kind == 2 ? (last_prefill ? 3 : 2) : A.commit_kind;
      commit_step<kMBlock>(c, kind, A.cand_lm, A.cand_exit, nwg, A.out_tokens, A.drafts, red, &bi[0][0]);
    }
    __syncthreads();
    if (tid == 0) grid_arrive(A.bar);
    nbar += 1;
    if (tid == 0) s_flag = grid_wait(A.bar, nbar * (unsigned)nwg, A.abort_flag) ? 1 : 0;
    __syncthreads();
    if (!s_flag) return;
  }
}

}  // namespace ppsd
