// Persistent-kernel engine: a whole ppsd_decode (or prefill) call in ONE cooperative launch.
//
// kMegaWgsPerCu workgroups of 512 threads per CU stay resident and walk the step's operations
// ("phases": QKV, attention, o_proj, gate/up, down of every layer, then the head) separated by
// grid barriers; a phase runs the same code as the corresponding per-operation kernel (same
// staging, same row-pair tasks, same attention unit), so both engines give bitwise equal results.
// The draft stage and the verify stage of a PPSD step are zipped: phase k runs operation k of
// BOTH stages (verify-while-draft, Sec. 4.2), the workgroups being divided between the two
// segments in proportion to their weight bytes, so a full step needs max(ops_draft, ops_verify)
// barriers instead of their sum.  Each workgroup stages exactly one input vector per phase.
//
// Every wait is bounded: a barrier that does not complete within kSpinLimit polls raises the
// abort flag, and every workgroup leaves the kernel at its next wait.
#pragma once

#include "ppsd_kernels.h"

namespace ppsd {

constexpr int kMBlock = 512;
constexpr int kMWaves = kMBlock / kWave;
constexpr int kMegaWgsPerCu = 2;
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
  int *cand_counts;    // [2]: candidates the LM / exit head phase of the current step produced
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

// ------------------------------------------------------------------------------------------
template <typename WT, int HD, int G>
__global__ __launch_bounds__(kMBlock, kMegaWgsPerCu) void k_mega(MegaArgs A) {
  extern __shared__ __align__(16) float lds[];            // one staged input vector; reused as the attention merge buffer
  __shared__ float red[kMWaves];
  __shared__ float bv[kMWaves];
  __shared__ int bi[kMWaves];
  __shared__ int s_flag;
  __shared__ int s_last;

  const Common &c = A.cm;
  const Dims &m = c.dm;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wg = blockIdx.x, nwg = gridDim.x;
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
    const int gen_row = uniform(vs->gen_count);
    const bool tracing = A.trace != nullptr && step == A.trace_step && wg == A.trace_wg && nph <= kTracePhases;

    auto slot_ptr = [&](int sel) -> float * {
      int slot = sel;
      if (sel == kHExitCur) slot = 2 + cur_h;
      else if (sel == kHExitNext) slot = 2 + (cur_h ^ 1);
      return c.xbuf + (size_t)slot * m.d;
    };

    // One weight-streaming segment on workgroups [wg0, wg0 + nw): stage its input, stream its tasks.
    auto run_stream = [&](const SegInfo &g, int si, const StageRun &run, int wg0, int nw) {
      const StageDesc &s = A.st[si];
      const LayerPtrs *lpp = A.layers + g.layer;
      const int gw = (wg - wg0) * kMWaves + wave, tw = nw * kMWaves;
      const bool first_layer = g.layer == s.lo, last_layer = g.layer == s.hi - 1;
      float *xs = lds;
      const WT *rows[kTripRows];
      Trip<WT, kTripRows, kTripBlocks> trip;
      if (g.kind == SK_QKV) {
        const WT *wqkv = (const WT *)uniform_ptr(lpp->wqkv);
        const int half = m.hd >> 1, d = m.d;
        auto set_rows = [&](int task) {
          const int head = task / half, i = task - head * half;
          rows[0] = wqkv + (size_t)(head * m.hd + i) * d;
          rows[1] = rows[0] + (size_t)half * d;
        };
        NormStage<WT, kMBlock> in;
        const bool emb = first_layer && s.from_embed;
        in.issue(emb ? nullptr : slot_ptr(first_layer ? s.xin_first : s.xwork),
                 emb ? (const WT *)A.embed + (size_t)run.tok * d : nullptr, uniform_ptr(lpp->attn_norm), d);
        if (gw < g.units) { set_rows(gw); trip_load<WT, kTripRows, kTripBlocks>(trip, rows, 0, col_blocks<WT>(d), d); }
        in.finish(d, m.eps, xs, red, (emb && wg == wg0) ? slot_ptr(s.xin_first) : nullptr);
        const int pos = run.pos;
        gemv_tasks<WT>(trip, rows, gw, g.units, tw, d, xs, set_rows, [&](int task, float lo, float hi) {
          if (lane != 0) return;
          const int h = task / half, i = task - h * half;
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
            WT *dst = kv_row<WT>(c, c.page_table, g.layer, pos, kvh, which);
            dst[i] = Pack<WT>::from_float(lo);
            dst[i + half] = Pack<WT>::from_float(hi);
          }
        });
      } else if (g.kind == SK_GATEUP) {
        const WT *wgu = (const WT *)uniform_ptr(lpp->wgu);
        const int d = m.d, f = m.f;
        auto set_rows = [&](int task) {
          rows[0] = wgu + (size_t)task * d;
          rows[1] = wgu + (size_t)(f + task) * d;
        };
        NormStage<WT, kMBlock> in;
        in.issue(slot_ptr(s.xwork), (const WT *)nullptr, uniform_ptr(lpp->mlp_norm), d);
        if (gw < f) { set_rows(gw); trip_load<WT, kTripRows, kTripBlocks>(trip, rows, 0, col_blocks<WT>(d), d); }
        in.finish(d, m.eps, xs, red, nullptr);
        float *mout = A.m[s.slot];
        gemv_tasks<WT>(trip, rows, gw, f, tw, d, xs, set_rows, [&](int task, float gt, float up) {
          if (lane == 0) mout[task] = gt / (1.0f + __expf(-gt)) * up;
        });
      } else if (g.kind == SK_OPROJ || g.kind == SK_DOWN) {
        const WT *W = (const WT *)uniform_ptr(g.kind == SK_OPROJ ? lpp->wo : lpp->wdown);
        const int C = g.C, n_rows = m.d;
        auto set_rows = [&](int task) {
          rows[0] = W + (size_t)(2 * task) * C;
          rows[1] = W + (size_t)min(2 * task + 1, n_rows - 1) * C;
        };
        CopyStage<kMBlock> in;
        in.issue(g.kind == SK_OPROJ ? A.a[s.slot] : A.m[s.slot], C);
        if (gw < g.units) { set_rows(gw); trip_load<WT, kTripRows, kTripBlocks>(trip, rows, 0, col_blocks<WT>(C), C); }
        in.template finish<WT>(C, xs);
        const float *resid = slot_ptr(g.kind == SK_OPROJ ? (first_layer ? s.xin_first : s.xwork) : s.xwork);
        float *out = slot_ptr(g.kind == SK_OPROJ ? s.xwork : (last_layer ? s.xout_last : s.xwork));
        gemv_tasks<WT>(trip, rows, gw, g.units, tw, C, xs, set_rows, [&](int task, float s0, float s1) {
          const int r = 2 * task + lane;
          if (lane < 2 && r < n_rows) out[r] = resid[r] + (lane == 0 ? s0 : s1);
        });
      } else {   // SK_HEAD
        const bool exit_head = s.head == 2;
        const WT *W = (const WT *)(exit_head ? A.exit_head : A.lm_head);
        const int d = m.d, V = m.V;
        auto set_rows = [&](int task) {
          rows[0] = W + (size_t)(2 * task) * d;
          rows[1] = W + (size_t)min(2 * task + 1, V - 1) * d;
        };
        NormStage<WT, kMBlock> in;
        in.issue(slot_ptr(s.head_xin), (const WT *)nullptr, exit_head ? A.exit_norm : A.final_norm, d);
        if (gw < g.units) { set_rows(gw); trip_load<WT, kTripRows, kTripBlocks>(trip, rows, 0, col_blocks<WT>(d), d); }
        in.finish(d, m.eps, xs, red, nullptr);
        float *lrow = nullptr;
        if (A.logits && !exit_head) {
          const int row = (s.role == kPrefill) ? 0 : gen_row;
          if (row < m.debug_rows) lrow = A.logits + (size_t)row * V;
        }
        float best = -INFINITY;
        int besti = kNoIndex;
        gemv_tasks<WT>(trip, rows, gw, g.units, tw, d, xs, set_rows, [&](int task, float s0, float s1) {
          const int r = 2 * task;
          if (better(s0, r, best, besti)) { best = s0; besti = r; }
          if (r + 1 < V && better(s1, r + 1, best, besti)) { best = s1; besti = r + 1; }
          if (lrow && lane == 0) { lrow[r] = s0; if (r + 1 < V) lrow[r + 1] = s1; }
        });
        if (lane == 0) { bv[wave] = best; bi[wave] = besti; }
        __syncthreads();
        if (tid == 0) {
          for (int w = 1; w < kMWaves; ++w)
            if (better(bv[w], bi[w], best, besti)) { best = bv[w]; besti = bi[w]; }
          float2 *cand = exit_head ? A.cand_exit : A.cand_lm;
          cand[wg - wg0] = make_float2(best, __int_as_float(besti));
          if (wg == wg0) A.cand_counts[exit_head ? 1 : 0] = nw;
        }
      }
    };

    // Attention segment on workgroups [wg0, wg0 + nw): units (kv head, split).
    auto run_attention = [&](const SegInfo &g, int si, const StageRun &run, int wg0, int nw) {
      const StageDesc &s = A.st[si];
      const int per = m.n_kv * A.attn_splits;
      for (int u = wg - wg0; u < per; u += nw) {
        const int kvh = u / A.attn_splits, split = u - kvh * A.attn_splits;
        attn_unit<WT, HD, G, kMBlock>(c, c.page_table, g.layer, run.pos, kvh, split, A.attn_splits, A.q[s.slot],
                                      A.a[s.slot], A.partials[s.slot], A.counters[s.slot], lds, &s_last);
      }
    };

    bool ok = true;
    for (int p = 0; p < nph && ok; ++p) {
      const PhaseSegs ps = phase_segs(A, p, run0, run1);
      if (!(ps.g0.active || ps.g1.active)) continue;
      // ---- wait for every workgroup to have finished the previous active phase
      if (nbar > 0) {
        if (tid == 0) s_flag = grid_wait(A.bar, nbar * (unsigned)nwg, A.abort_flag) ? 1 : 0;
        __syncthreads();
        if (!s_flag) { ok = false; break; }
      }
      if (tracing && tid == 0) A.trace[p * kTraceSlots + 0] = wall_clock64();
      // ---- divide the workgroups between the two segments in proportion to their weight bytes
      int n0 = nwg;
      if (ps.g0.active && ps.g1.active) {
        const long long b0 = ps.g0.kind == SK_ATTN ? 1 : (long long)ps.g0.units * ps.g0.C;
        const long long b1 = ps.g1.kind == SK_ATTN ? 1 : (long long)ps.g1.units * ps.g1.C;
        n0 = (int)((b0 * nwg + (b0 + b1) / 2) / (b0 + b1));
        n0 = max(1, min(nwg - 1, n0));
      } else if (!ps.g0.active) {
        n0 = 0;
      }
      if (wg < n0) {
        const StageRun &r = ps.s0 ? run1 : run0;
        if (ps.g0.kind == SK_ATTN) run_attention(ps.g0, ps.s0, r, 0, n0);
        else run_stream(ps.g0, ps.s0, r, 0, n0);
      } else {
        if (ps.g1.kind == SK_ATTN) run_attention(ps.g1, ps.s1, run1, n0, nwg - n0);
        else run_stream(ps.g1, ps.s1, run1, n0, nwg - n0);
      }
      // ---- arrive
      __syncthreads();
      if (tracing && tid == 0) A.trace[p * kTraceSlots + 2] = wall_clock64();
      if (tid == 0) {
        grid_arrive(A.bar);
        if (tracing) A.trace[p * kTraceSlots + 3] = wall_clock64();
      }
      nbar += 1;
    }
    if (!ok) return;

    // ---- commit: everyone waits for the last phase, workgroup 0 commits, everyone waits for that
    if (tid == 0) s_flag = grid_wait(A.bar, nbar * (unsigned)nwg, A.abort_flag) ? 1 : 0;
    __syncthreads();
    if (!s_flag) return;
    if (wg == 0) {
      // a head segment wrote one candidate per workgroup it ran on (see the division above)
      const int kind = A.commit_kind == 2 ? (last_prefill ? 3 : 2) : A.commit_kind;
      volatile const int *cc = A.cand_counts;
      commit_step<kMBlock>(c, kind, A.cand_lm, uniform(cc[0]), A.cand_exit, uniform(cc[1]), A.out_tokens, A.drafts, red, bi);
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
