// Host side of the C ABI declared in include/ppsd.h: context, workspace layout, the one-GPU
// step scheduler (draft stage and verify stage on two streams, one commit kernel per step,
// optionally replayed from a captured HIP graph) and the decode loop.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "../../include/ppsd.h"
#include "ppsd_mega.h"
#include "ppsd_prefill.h"
#include "ppsd_batch.h"

using namespace ppsd;

static __device__ __align__(256) unsigned char scratch[PPSD_STATIC_SCRATCH_BYTES];

namespace {

thread_local std::string g_err;

int fail(int code, const char *fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  g_err = buf;
  return code;
}

#define HIP_TRY(expr)                                                                     \
  do {                                                                                    \
    hipError_t e_ = (expr);                                                               \
    if (e_ != hipSuccess) return fail(PPSD_EHIP, "%s: %s", #expr, hipGetErrorString(e_)); \
  } while (0)

constexpr size_t kAlign = 256;
size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

constexpr int kOneSplitUpTo = 512;     // attention: a single split up to this capacity (max_seq)
constexpr int kSplitPositions = 512;   // beyond it, one split per this many positions of capacity at least; at load
                                       // the count is raised until the attention workgroups fill the chip once
                                       // (8704 positions, 8 KV heads: 24 / 32 / 40 / 56 splits -> 19.0 / 18.3 / 24.1 / 21.2 us)
constexpr int kMaxSplits = kMaxAttnSplits;   // attention splits along the sequence (both engines)
constexpr int kDefaultGamma = 3;       // drafts per round of PPSD_MODE_EESD
constexpr size_t kBatchLdsMax = 150 * 1024;   // staged input vectors of a batched kernel: at most this much LDS
constexpr size_t kBatchSlabBytes = 64 * 1024; // o_proj / down of the batched pass: column slabs of at most this much
constexpr int kMaxStreams = 4;         // streams the stages of a pipeline tick are spread over

enum Kind { kKQkv = 0, kKAttn, kKOproj, kKGateUp, kKDown, kKHead, kKCommit };

// The per-step scratch region of ppsd_decode_static_scratch.  In host code the array's name is only a
// stand-in; its device address is taken once per device with hipGetSymbolAddress (ppsd_load_weights does
// it for the current device) and kept here.  Every device holds its own copy until the process ends.
constexpr int kMaxDevices = 64;
void *g_static_scratch[kMaxDevices] = {};

struct Layout {
  size_t state, prompt, out_tokens, drafts, page_table, rope_cos, rope_sin, xbuf;
  size_t q[kMaxStreams], a[kMaxStreams], mbuf[kMaxStreams], partials[kMaxStreams], counters[kMaxStreams], cand_lm, cand_exit, sink, logits, kv;
  size_t layer_ptrs, bar, abort_flag, trace, cand_counts;
  size_t pf_x, pf_q, pf_ao, pf_ah, pf_al, pf_mh, pf_ml, pf_part;   // MFMA prefill chunk buffers (0 bytes when not used)
  int pf_chunk;          // positions per prefill chunk
  size_t qb, ab, mb, partials_b, counters_b, cand_b;   // batched verify pass (0 bytes unless PPSD_MODE_EESD)
  size_t logits_lm, logits_exit, probs;                // sampling (0 bytes unless temperature > 0)
  size_t logits_b, probs_e;                            // sampling in draft-then-verify rounds
  bool pf;
  size_t scratch0, scratch_bytes;                      // the per-step scratch region [scratch0, scratch0 + scratch_bytes)
  size_t total;
  int n_pages, n_splits, head_blocks;
};

// Stages of the full pipeline schedule: stage 0 is the draft model (layers 1..E); the layers behind it are cut
// into stages of pipeline_stage_layers layers each (0 = E, the balanced partition of Sec. 4.1), the last taking
// what remains.
int later_stage_layers(const ppsd_config *c) { return c->pipeline_stage_layers > 0 ? c->pipeline_stage_layers : c->exit_layer; }
int pipeline_stages(const ppsd_config *c) {
  const int w = later_stage_layers(c);
  return 1 + (c->n_layers - c->exit_layer + w - 1) / w;
}

bool valid_config(const ppsd_config *c, const char **why) {
#define REJECT(cond, msg) if (cond) { *why = msg; return false; }
  REJECT(!c, "null config");
  REJECT(c->n_layers < 2 || c->exit_layer < 1 || c->exit_layer >= c->n_layers, "need 1 <= exit_layer < n_layers");
  REJECT(c->head_dim != 64 && c->head_dim != 128, "head_dim must be 64 or 128");
  REJECT(c->n_heads < 1 || c->n_kv_heads < 1 || c->n_heads % c->n_kv_heads, "n_heads must be a multiple of n_kv_heads");
  const int g = c->n_kv_heads ? c->n_heads / c->n_kv_heads : 0;
  REJECT(g != 1 && g != 2 && g != 4, "n_heads / n_kv_heads must be 1, 2 or 4");
  REJECT(c->dtype != PPSD_FP32 && c->dtype != PPSD_BF16, "dtype must be PPSD_FP32 or PPSD_BF16");
  const int vec = c->dtype == PPSD_FP32 ? 4 : 8;
  REJECT(c->d_model < vec || c->d_model % vec, "d_model must be a multiple of the 16-byte vector width");
  REJECT(c->d_ffn < vec || c->d_ffn % vec, "d_ffn must be a multiple of the 16-byte vector width");
  REJECT(c->vocab < 2, "vocab too small");
  REJECT(c->max_seq < 3, "max_seq too small");
  REJECT(c->kv_page_tokens != 8 && c->kv_page_tokens != 16 && c->kv_page_tokens != 32 && c->kv_page_tokens != 64,
         "kv_page_tokens must be 8, 16, 32 or 64");
  REJECT((double)(c->n_layers + 1) * ((c->max_seq + c->kv_page_tokens - 1) / c->kv_page_tokens) * c->n_kv_heads * 2 >= 2147483648.0,
         "layers x pages x KV heads x 2 must stay below 2^31 (KV block index)");
  REJECT(c->mode < 0 || c->mode > 4, "mode must be 0..4");
  REJECT(!(c->rope_base > 1.0f) || !(c->rms_eps >= 0.0f), "bad rope_base / rms_eps");
  REJECT(c->debug_logits < 0, "debug_logits < 0");
  const int esz = c->dtype == PPSD_FP32 ? 4 : 2;
  REJECT((size_t)xs_floats(esz, c->d_ffn) * 4 > 64 * 1024 || (size_t)xs_floats(esz, c->d_model) * 4 > 64 * 1024 ||
         (size_t)xs_floats(esz, c->n_heads * c->head_dim) * 4 > 64 * 1024, "activation vector exceeds 64 KiB of LDS");
  REJECT(c->d_model > 16 * kGBlock, "d_model exceeds the staging capacity (8192)");
  REJECT(c->d_ffn > 32 * kGBlock || c->n_heads * c->head_dim > 32 * kGBlock, "d_ffn / n_heads*head_dim exceed the staging capacity (16384)");
  REJECT(c->engine != PPSD_ENGINE_STREAMS && c->engine != PPSD_ENGINE_PERSISTENT, "engine must be 0 or 1");
  REJECT(c->engine == PPSD_ENGINE_PERSISTENT && c->time_kernels, "time_kernels needs the per-operation engine");
  REJECT(c->prefill_loop != 0 && c->prefill_loop != 1, "prefill_loop must be 0 or 1");
  REJECT(c->prefill_chunk != 0 && (c->prefill_chunk < kPfBM || c->prefill_chunk > kPfChunkMax || c->prefill_chunk % kPfBM),
         "prefill_chunk must be 0 or a multiple of 128 in 128..4096");
  REJECT(c->tune_prefill_tile < 0 || c->tune_prefill_tile > 2, "tune_prefill_tile must be 0, 1 or 2");
  if (c->mode == PPSD_MODE_PIPELINE) {
    REJECT(c->engine != PPSD_ENGINE_STREAMS, "the full pipeline schedule runs on the per-operation engine only");
    REJECT(c->time_kernels, "time_kernels is not available with the full pipeline schedule");
    REJECT(c->pipeline_stage_layers < 0 || c->pipeline_stage_layers > c->n_layers, "pipeline_stage_layers must be 0 (= exit_layer) or 1..n_layers");
    REJECT(pipeline_stages(c) > kMaxStages, "more than 16 pipeline stages (n_layers / exit_layer)");
  }
  REJECT(c->pipeline_streams < 0 || c->pipeline_streams == 1 || c->pipeline_streams > kMaxStreams, "pipeline_streams must be 0 (default) or 2..4");
  REJECT(c->tune_wgs_per_cu < 0 || c->tune_wgs_per_cu > 4, "tune_wgs_per_cu must be 0..4");
  REJECT(c->tune_draft_share < 0 || c->tune_draft_share > 100, "tune_draft_share must be 0 (default) or 1..100 percent");
  REJECT(c->eesd_gamma < 0 || c->eesd_gamma > kMaxGamma, "eesd_gamma must be 0 (default) or 1..4");
  if (c->mode == PPSD_MODE_EESD) {
    REJECT(c->engine != PPSD_ENGINE_STREAMS, "draft-then-verify rounds run on the per-operation engine only");
    REJECT(c->time_kernels, "time_kernels is not available with draft-then-verify rounds");
    const int B = (c->eesd_gamma ? c->eesd_gamma : kDefaultGamma) + 1;
    REJECT((size_t)B * xs_floats(esz, c->d_model) * 4 > kBatchLdsMax, "gamma + 1 input vectors of d_model floats exceed the LDS of a compute unit");
  }
  REJECT(c->tune_attn_split < 0 || (c->tune_attn_split > 0 && c->tune_attn_split < 64), "tune_attn_split must be 0 or >= 64");
  REJECT(!(c->temperature >= 0.0f) || c->temperature > 1.0e4f, "temperature must be in [0, 1e4] (0 = greedy)");
  REJECT(c->temperature > 0.0f && c->temperature < 1.0e-4f, "a positive temperature must be at least 1e-4");
  REJECT(c->temperature > 0.0f && (c->engine != PPSD_ENGINE_STREAMS || c->time_kernels),
         "sampling (temperature > 0) runs on the per-operation engine, without time_kernels");
  REJECT(c->exit_block != 0 && c->exit_block != 1, "exit_block must be 0 or 1");
  REJECT(c->exit_block && c->engine == PPSD_ENGINE_PERSISTENT, "the transformer-layer exit head runs on the per-operation engine only");
  REJECT(c->exit_block && c->time_kernels, "time_kernels is not available with the transformer-layer exit head");
#undef REJECT
  return true;
}

// The matrix-core prefill covers bf16 storage, head_dim 128 and tile-aligned widths.
bool pf_eligible(const ppsd_config *c) {
  return !c->prefill_loop && c->dtype == PPSD_BF16 && c->head_dim == 128 && c->d_model % kPfBN == 0 && c->d_ffn % 64 == 0 &&
         c->d_model % kPfBK == 0 && c->d_ffn % kPfBK == 0;
}

Layout make_layout(const ppsd_config *c) {
  Layout L{};
  const size_t es = c->dtype == PPSD_FP32 ? 4 : 2;
  L.n_pages = (c->max_seq + c->kv_page_tokens - 1) / c->kv_page_tokens;
  const int per_split = c->tune_attn_split > 0 ? c->tune_attn_split : kSplitPositions;
  int ns = c->max_seq <= kOneSplitUpTo && c->tune_attn_split == 0 ? 1 : (c->max_seq + per_split - 1) / per_split;
  L.n_splits = ns < 1 ? 1 : (ns > kMaxSplits ? kMaxSplits : ns);
  L.head_blocks = kMaxWorkgroups;   // capacity of the candidate arrays; the live count is set at load
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
  L.state = take(sizeof(DevState));
  L.prompt = take(4ull * c->max_seq);
  L.out_tokens = take(4ull * c->max_seq);
  L.drafts = take(4ull * (c->max_seq + 1));
  L.page_table = take(4ull * L.n_pages);
  L.rope_cos = take(4ull * c->max_seq * (c->head_dim / 2));
  L.rope_sin = take(4ull * c->max_seq * (c->head_dim / 2));
  L.xbuf = take(4ull * kXSlots * c->d_model);
  const size_t nq = (size_t)c->n_heads * c->head_dim;
  // Per-step scratch, one contiguous region: vectors between the kernels of a layer, attention split
  // partials and their arrival counters, the heads' candidates, the batched pass's vectors.  Nothing in it
  // outlives a step (the counters are back at zero after every use), so ppsd_decode_static_scratch can
  // run the same kernels with this region in the library's static device array instead.
  L.scratch0 = off;
  for (int s = 0; s < kMaxStreams; ++s) {
    L.q[s] = take(4 * nq);
    L.a[s] = take(4 * nq);
    L.mbuf[s] = take(4ull * c->d_ffn);
    L.partials[s] = take(4ull * c->n_heads * kMaxSplits * (c->head_dim + 2));
    L.counters[s] = take(4ull * kCounterStride * c->n_kv_heads);
  }
  const size_t n_cand = kMaxWorkgroups;
  L.cand_lm = take(8ull * n_cand);
  L.cand_exit = take(8ull * n_cand);
  const size_t nb = c->mode == PPSD_MODE_EESD ? kMaxBatch : 0;
  L.qb = take(4ull * nb * nq);
  L.ab = take(4ull * nb * nq);
  L.mb = take(4ull * nb * c->d_ffn);
  L.partials_b = take(4ull * nb * c->n_heads * kMaxSplits * (c->head_dim + 2));
  L.counters_b = take(4ull * nb * kCounterStride * c->n_kv_heads);
  L.cand_b = take(8ull * nb * n_cand);
  L.scratch_bytes = off - L.scratch0;
  L.layer_ptrs = take(sizeof(LayerPtrs) * (size_t)c->n_layers);
  L.bar = take(256);
  L.abort_flag = take(256);
  L.cand_counts = take(256);
  L.trace = take(8ull * kTraceSlots * kTracePhases);
  L.pf = pf_eligible(c);
  // a chunk covers the whole prompt when max_seq allows, 4096 positions at most
  L.pf_chunk = !L.pf ? 0 : c->prefill_chunk ? c->prefill_chunk : std::min(kPfChunkMax, (c->max_seq + kPfBM - 1) / kPfBM * kPfBM);
  const size_t pc = (size_t)L.pf_chunk;
  const size_t wide = std::max((size_t)c->d_model, nq);
  L.pf_x = take(4ull * pc * c->d_model);
  L.pf_q = take(4ull * pc * nq);
  L.pf_ao = take(4ull * pc * nq);
  L.pf_ah = take(2ull * pc * wide);
  L.pf_al = take(2ull * pc * wide);
  L.pf_mh = take(2ull * pc * c->d_ffn);
  L.pf_ml = take(2ull * pc * c->d_ffn);
  size_t part = 0;       // the largest split-K partial-sum buffer any chunk length can ask for
  const int tile = c->tune_prefill_tile ? c->tune_prefill_tile : -1;
  for (int nv = kPfBM; nv <= L.pf_chunk; nv += kPfBM) {
    part = std::max(part, pf_partial_floats(pf_plan(nv, (int)(nq + 2ull * c->n_kv_heads * c->head_dim), c->d_model, tile)));
    part = std::max(part, pf_partial_floats(pf_plan(nv, c->d_model, (int)nq, tile)));
    part = std::max(part, pf_partial_floats(pf_plan(nv, 2 * c->d_ffn, c->d_model, tile)));
    part = std::max(part, pf_partial_floats(pf_plan(nv, c->d_model, c->d_ffn, tile)));
  }
  L.pf_part = take(4ull * part);
  const size_t nv = c->temperature > 0.0f ? (size_t)c->vocab : 0;
  L.logits_lm = take(4ull * nv);
  L.logits_exit = take(4ull * nv);
  L.probs = take(4ull * (c->mode == PPSD_MODE_PIPELINE ? kMaxStages : 2) * nv);
  const size_t nve = c->mode == PPSD_MODE_EESD ? nv : 0;
  L.logits_b = take(4ull * kMaxBatch * nve);
  L.probs_e = take(4ull * kMaxGamma * nve);
  L.sink = take(256);
  L.logits = take(4ull * c->debug_logits * c->vocab);
  L.kv = take((size_t)(c->n_layers + c->exit_block) * L.n_pages * c->n_kv_heads * 2 * c->kv_page_tokens * c->head_dim * es);
  L.total = off;
  return L;
}

}  // namespace

struct ppsd_ctx {
  ppsd_config cfg;
  Layout lay;
  Common cm;
  const void *embed, *final_norm, *lm_head, *exit_norm, *exit_head;
  std::vector<const void *> attn_norm, wqkv, wo, mlp_norm, wgu, wdown;
  char *ws;
  char *scr = nullptr;                  // base of the per-step scratch region: ws + lay.scratch0, or the static array
  int32_t *h_out = nullptr;             // pinned, max_seq ints: staging of the committed tokens on their way to the host
  hipStream_t sA, sB;
  hipStream_t sx[kMaxStreams] = {};     // pipeline ticks: sx[0] = sA, sx[1] = sB, the rest created here
  int n_streams = 2;
  int gamma = 0;                        // drafts per round (PPSD_MODE_EESD)
  hipEvent_t ev_fork, ev_join, ev_t0, ev_t1;
  hipEvent_t ev_joinx[kMaxStreams] = {};
  hipGraphExec_t g_step = nullptr;      // decode step in cfg.mode
  hipGraphExec_t g_prefill = nullptr;   // one prompt position, no head
  DevState *h_state = nullptr;          // pinned
  // persistent engine
  int n_cu = 0;                         // compute units of the device
  int device = -1;                      // the device the context was created on
  int n_wg = 0;
  // bytes of LDS a staged input vector of C elements takes (padded to whole column blocks)
  size_t xs_bytes(int C) const { return 4ull * xs_floats(cfg.dtype == PPSD_FP32 ? 4 : 2, C); }
  // grid of a weight-streaming kernel with n_tasks row-pair tasks: one wave per task up to a few
  // workgroups per CU, then the waves loop
  int gemv_grid(int n_tasks, int wgs_per_cu = kGemvWgsPerCu) const {
    return gemv_grid_for(n_tasks, n_cu, cfg.tune_wgs_per_cu > 0 ? cfg.tune_wgs_per_cu : wgs_per_cu);
  }
  int xs_stride = 0;
  size_t mega_lds = 0;
  int trace_step = -1, trace_wg = 0;
  bool prefilled = false;
  int host_len = 0;                     // prompt length + tokens committed so far (token #0 included)
  int64_t steps_launched = 0;
  double device_ms = 0.0;
  // profiling mode
  std::vector<hipEvent_t> tk_events;
  std::vector<int> tk_kinds;
  size_t tk_used = 0;
  ppsd_kernel_times_t ktimes{};
};

namespace {

template <typename T> T *at(ppsd_ctx *x, size_t off) { return reinterpret_cast<T *>(x->ws + off); }
// a buffer of the per-step scratch region, wherever that region lives for the running call
template <typename T> T *sc(ppsd_ctx *x, size_t off) { return reinterpret_cast<T *>(x->scr + (off - x->lay.scratch0)); }

// Launch helper.  In profiling mode (all launches on one stream) one event is recorded at the start
// of the step and one after every kernel: kernel i lasted from event i to event i + 1.  A single
// event between two kernels keeps what the measurement adds to a launch near 1 us (an event pair
// around every launch added 2-3 us).
struct Launcher {
  ppsd_ctx *x;
  hipStream_t s;
  bool timed;
  hipError_t err = hipSuccess;

  void need_event(size_t idx) {
    while (err == hipSuccess && x->tk_events.size() <= idx) {
      hipEvent_t e;
      err = hipEventCreate(&e);
      if (err == hipSuccess) x->tk_events.push_back(e);
    }
  }
  void before(int kind) {
    if (!timed || err != hipSuccess) return;
    if (x->tk_used == 0) {
      need_event(0);
      if (err != hipSuccess) return;
      err = hipEventRecord(x->tk_events[0], s);
      x->tk_used = 1;
    }
    x->tk_kinds.resize(x->tk_used);
    x->tk_kinds[x->tk_used - 1] = kind;
  }
  void after() {
    if (err == hipSuccess) err = hipGetLastError();
    if (!timed || err != hipSuccess) return;
    need_event(x->tk_used);
    if (err != hipSuccess) return;
    err = hipEventRecord(x->tk_events[x->tk_used], s);
    x->tk_used += 1;
  }
};

// Trips a wave of a weight-streaming kernel keeps in flight: two where several kernel chains share the chip
// (the stages of the pipeline schedule), one for a single chain or two chains.
inline bool deep_role(int role) { return role >= kPipeStage0 && role < kEesdDraft0; }
constexpr int kDeepWgsPerCu = 2;      // what stays resident at the deeper variant's register count

template <typename WT>
void launch_layer(Launcher &L, int role, int layer, int stage, int xin_sel, int xout_last_sel, bool from_embed, int xwork) {
  ppsd_ctx *x = L.x;
  const ppsd_config &c = x->cfg;
  const Common &cm = x->cm;
  const int d = c.d_model, f = c.d_ffn, nq = c.n_heads * c.head_dim;
  float *q = sc<float>(x, x->lay.q[stage]);
  float *a = sc<float>(x, x->lay.a[stage]);
  float *mb = sc<float>(x, x->lay.mbuf[stage]);
  // xwork: residual slot used inside the layer after the first residual add
  const int total_pairs = (c.n_heads + 2 * c.n_kv_heads) * (c.head_dim / 2);
  const bool deep = deep_role(role);
  L.before(kKQkv);
  if (deep)
    hipLaunchKernelGGL((k_qkv<WT, 2>), dim3(x->gemv_grid(total_pairs, kDeepWgsPerCu)), dim3(kGBlock), x->xs_bytes(d), L.s, cm, role, layer,
                       xin_sel, from_embed ? 1 : 0, (const WT *)x->embed, (const float *)x->attn_norm[layer],
                       (const WT *)x->wqkv[layer], q);
  else
    hipLaunchKernelGGL((k_qkv<WT, 1>), dim3(x->gemv_grid(total_pairs)), dim3(kGBlock), x->xs_bytes(d), L.s, cm, role, layer,
                       xin_sel, from_embed ? 1 : 0, (const WT *)x->embed, (const float *)x->attn_norm[layer],
                       (const WT *)x->wqkv[layer], q);
  L.after();

  const dim3 agrid(c.n_kv_heads, x->lay.n_splits);
  float *part = sc<float>(x, x->lay.partials[stage]);
  int *cnt = sc<int>(x, x->lay.counters[stage]);
  const int G = c.n_heads / c.n_kv_heads;
  L.before(kKAttn);
#define ATTN(HD, GG) hipLaunchKernelGGL((k_attn<WT, HD, GG>), agrid, dim3(kGBlock), 0, L.s, cm, role, layer, \
                                        (const float *)q, a, part, cnt)
  if (c.head_dim == 64) { if (G == 1) ATTN(64, 1); else if (G == 2) ATTN(64, 2); else ATTN(64, 4); }
  else { if (G == 1) ATTN(128, 1); else if (G == 2) ATTN(128, 2); else ATTN(128, 4); }
#undef ATTN
  L.after();

  const int proj_grid = x->gemv_grid(d, deep ? kDeepWgsPerCu : kGemvWgsPerCu);   // one row per task
  L.before(kKOproj);
  if (deep)
    hipLaunchKernelGGL((k_proj_resid<WT, 2>), dim3(proj_grid), dim3(kGBlock), x->xs_bytes(nq), L.s, cm, role,
                       (const float *)a, nq, (const WT *)x->wo[layer], d, xin_sel, xwork);
  else
    hipLaunchKernelGGL((k_proj_resid<WT, 1>), dim3(proj_grid), dim3(kGBlock), x->xs_bytes(nq), L.s, cm, role,
                       (const float *)a, nq, (const WT *)x->wo[layer], d, xin_sel, xwork);
  L.after();

  L.before(kKGateUp);
  if (deep)
    hipLaunchKernelGGL((k_gate_up<WT, 2>), dim3(x->gemv_grid(f, kGateUpWgsPerCu)), dim3(kGBlock), x->xs_bytes(d), L.s, cm, role, xwork,
                       (const float *)x->mlp_norm[layer], (const WT *)x->wgu[layer], mb);
  else
    hipLaunchKernelGGL((k_gate_up<WT, 1>), dim3(x->gemv_grid(f, kGateUpWgsPerCu)), dim3(kGBlock), x->xs_bytes(d), L.s, cm, role, xwork,
                       (const float *)x->mlp_norm[layer], (const WT *)x->wgu[layer], mb);
  L.after();

  L.before(kKDown);
  // An input vector of which three workgroups per compute unit cannot each stage a whole copy, under a grid that
  // then no longer fits the chip in one round (13B: 640 workgroups, two per compute unit): two column slabs.
  // Where the grid fits anyway (8B: 512 workgroups) the whole vector is staged: one barrier less.
  const int fit_whole = (int)((160 * 1024) / (x->xs_bytes(f) + 1024));
  if (f > kSlabAbove && proj_grid > fit_whole * x->n_cu) {
    const int blk = kWave * (16 / (int)sizeof(WT));
    const int Cs = ((f + 1) / 2 + blk - 1) / blk * blk;
    if (deep)
      hipLaunchKernelGGL((k_proj_resid_slabs<WT, 2>), dim3(proj_grid), dim3(kGBlock), x->xs_bytes(Cs), L.s, cm, role,
                         (const float *)mb, f, Cs, (const WT *)x->wdown[layer], d, xwork, xout_last_sel);
    else
      hipLaunchKernelGGL((k_proj_resid_slabs<WT, 1>), dim3(proj_grid), dim3(kGBlock), x->xs_bytes(Cs), L.s, cm, role,
                         (const float *)mb, f, Cs, (const WT *)x->wdown[layer], d, xwork, xout_last_sel);
  } else if (deep)
    hipLaunchKernelGGL((k_proj_resid<WT, 2>), dim3(proj_grid), dim3(kGBlock), x->xs_bytes(f), L.s, cm, role,
                       (const float *)mb, f, (const WT *)x->wdown[layer], d, xwork, xout_last_sel);
  else
    hipLaunchKernelGGL((k_proj_resid<WT, 1>), dim3(proj_grid), dim3(kGBlock), x->xs_bytes(f), L.s, cm, role,
                       (const float *)mb, f, (const WT *)x->wdown[layer], d, xwork, xout_last_sel);
  L.after();
}

template <typename WT>
void launch_head(Launcher &L, int role, int xin_sel, bool is_lm) {
  ppsd_ctx *x = L.x;
  const ppsd_config &c = x->cfg;
  float2 *cand = sc<float2>(x, is_lm ? x->lay.cand_lm : x->lay.cand_exit);
  float *logits = c.debug_logits > 0 ? at<float>(x, x->lay.logits) : nullptr;
  float *full = c.temperature > 0.0f ? at<float>(x, is_lm ? x->lay.logits_lm : x->lay.logits_exit) : nullptr;
  L.before(kKHead);
  // the commit kernels read head_blocks candidates: both variants launch that many workgroups (the deeper one
  // keeps two of them resident per compute unit and runs the rest behind them)
  if (deep_role(role))
    hipLaunchKernelGGL((k_head<WT, 2>), dim3(x->cm.dm.head_blocks), dim3(kGBlock), x->xs_bytes(c.d_model), L.s,
                       x->cm, role, xin_sel, (const float *)(is_lm ? x->final_norm : x->exit_norm),
                       (const WT *)(is_lm ? x->lm_head : x->exit_head), cand, logits, is_lm ? 1 : 0, full);
  else
    hipLaunchKernelGGL((k_head<WT, 1>), dim3(x->cm.dm.head_blocks), dim3(kGBlock), x->xs_bytes(c.d_model), L.s,
                       x->cm, role, xin_sel, (const float *)(is_lm ? x->final_norm : x->exit_norm),
                       (const WT *)(is_lm ? x->lm_head : x->exit_head), cand, logits, is_lm ? 1 : 0, full);
  L.after();
}

void launch_commit(Launcher &L, int kind) {
  ppsd_ctx *x = L.x;
  if (x->cfg.temperature > 0.0f && kind != 2) {   // sampling: kinds 0 (vanilla), 1 (two-stage step), 3 (token #0), 4 (tick)
    L.before(kKCommit);
    hipLaunchKernelGGL(k_commit_sample, dim3(1), dim3(kSBlock), 0, L.s, x->cm, kind, at<const float>(x, x->lay.logits_lm),
                       at<const float>(x, x->lay.logits_exit), at<float>(x, x->lay.probs), 1.0f / x->cfg.temperature,
                       (uint32_t)x->cfg.sample_seed, at<int32_t>(x, x->lay.out_tokens), at<int32_t>(x, x->lay.drafts));
    L.after();
    return;
  }
  L.before(kKCommit);
  hipLaunchKernelGGL(k_commit, dim3(1), dim3(kBlock), 0, L.s, x->cm, kind, sc<const float2>(x, x->lay.cand_lm),
                     sc<const float2>(x, x->lay.cand_exit), at<int32_t>(x, x->lay.out_tokens),
                     at<int32_t>(x, x->lay.drafts));
  L.after();
}

// A stage = a run of layers [lo, hi) for one role.  The first layer reads xin_first (or the
// embedding); the last layer's down-projection writes xout_last; xwork (a fixed-address slot)
// carries the residual stream in between.  `stage` picks the set of scratch vectors (q, attention
// output, MLP activation, split partials): stages that may run concurrently need different sets.
template <typename WT>
void launch_stage(Launcher &L, int role, int lo, int hi, int stage, int xin_first, bool from_embed, int xout_last,
                  int xwork = -1) {
  if (xwork < 0) xwork = (role == kVerify) ? kXVerify : kXDraft;
  for (int l = lo; l < hi; ++l)
    launch_layer<WT>(L, role, l, stage, l == lo ? xin_first : xwork, l == hi - 1 ? xout_last : xwork,
                     from_embed && l == lo, xwork);
}

// The transformer-layer early-exit head (Sec. 5.4): entry n_layers of the per-layer weights, run on
// the layer-E hidden state in slot xin; its output (slot xwork) feeds the exit head only.  With
// kv_only just its K/V row is appended (positions whose draft nobody needs: the prompt, the last
// draft of a draft-then-verify round) -- later drafts attend to it.
template <typename WT>
void launch_exit_block(Launcher &L, int role, int stage, int xin, int xwork, bool kv_only) {
  ppsd_ctx *x = L.x;
  const ppsd_config &c = x->cfg;
  const int layer = c.n_layers;
  if (!kv_only) {
    launch_layer<WT>(L, role, layer, stage, xin, xwork, false, xwork);
    return;
  }
  const int total_pairs = (c.n_heads + 2 * c.n_kv_heads) * (c.head_dim / 2);
  L.before(kKQkv);
  hipLaunchKernelGGL((k_qkv<WT, 1>), dim3(x->gemv_grid(total_pairs)), dim3(kGBlock), x->xs_bytes(c.d_model), L.s, x->cm, role,
                     layer, xin, 0, (const WT *)x->embed, (const float *)x->attn_norm[layer], (const WT *)x->wqkv[layer],
                     sc<float>(x, x->lay.q[stage]));
  L.after();
}

// ---------------------------------------------------------------- draft-then-verify round
// Workgroups of a batched kernel: as many as stay resident with `lds` bytes of staged input each.
int batch_grid(const ppsd_ctx *x, int n_tasks, size_t lds, int wgs_per_cu) {
  int fit = (int)((160 * 1024) / (lds + 1024));
  if (fit < 1) fit = 1;
  if (fit < wgs_per_cu) wgs_per_cu = fit;
  return x->gemv_grid(n_tasks, wgs_per_cu);
}

template <typename WT, int B>
void launch_proj_b(Launcher &L, int kind, const float *vin, int C, const WT *W, int resid_slot0, int out_slot0) {
  ppsd_ctx *x = L.x;
  const int d = x->cfg.d_model;
  int Cs = C;                                           // one slab when the B staged vectors fit the slab budget
  if ((size_t)B * C * 4 > kBatchSlabBytes) {
    // The slab-walking kernel has one row per wave: size the slabs so that all its workgroups are resident at
    // once, two per compute unit or, with more rows than that, three (its registers allow three).
    const int blk = 512;                                // slabs end on column-block boundaries
    const int wgs = (d + kGWaves - 1) / kGWaves;
    const int per_cu = wgs > 2 * x->n_cu ? 3 : 2;
    size_t budget = (size_t)160 * 1024 / per_cu - 2048;
    if (budget > kBatchSlabBytes) budget = kBatchSlabBytes;
    int cs_max = (int)(budget / 4 / B) / blk * blk;
    if (cs_max < blk) cs_max = blk;
    const int n_slabs = (C + cs_max - 1) / cs_max;
    Cs = ((C + n_slabs - 1) / n_slabs + blk - 1) / blk * blk;
  }
  if (Cs < C) {
    // several slabs: one launch that walks them, one row per wave
    L.before(kind);
    hipLaunchKernelGGL((k_proj_resid_bs<WT, B>), dim3((d + kGWaves - 1) / kGWaves), dim3(kGBlock), (size_t)B * x->xs_bytes(Cs), L.s, x->cm,
                       vin, C, Cs, W, d, resid_slot0, out_slot0);
    L.after();
    return;
  }
  const size_t lds = (size_t)B * x->xs_bytes(C);
  L.before(kind);
  hipLaunchKernelGGL((k_proj_resid_b<WT, B>), dim3(batch_grid(x, (d + 1) / 2, lds, kGemvWgsPerCu)), dim3(kGBlock), lds, L.s, x->cm, vin,
                     C, 0, C, W, d, resid_slot0, out_slot0);
  L.after();
}

template <typename WT, int B>
void launch_verify_batch(Launcher &L) {
  ppsd_ctx *x = L.x;
  const ppsd_config &c = x->cfg;
  const Common &cm = x->cm;
  const int d = c.d_model, f = c.d_ffn, nq = c.n_heads * c.head_dim;
  float *q = sc<float>(x, x->lay.qb), *a = sc<float>(x, x->lay.ab), *mb = sc<float>(x, x->lay.mb);
  float *part = sc<float>(x, x->lay.partials_b);
  int *cnt = sc<int>(x, x->lay.counters_b);
  const size_t lds_d = (size_t)B * x->xs_bytes(d);
  const int total_pairs = (c.n_heads + 2 * c.n_kv_heads) * (c.head_dim / 2);
  const int G = c.n_heads / c.n_kv_heads;
  for (int l = c.exit_layer; l < c.n_layers; ++l) {
    const int xin0 = l == c.exit_layer ? kXBatchInSlot0 : kXBatchWorkSlot0;
    L.before(kKQkv);
    hipLaunchKernelGGL((k_qkv_b<WT, B>), dim3(batch_grid(x, total_pairs, lds_d, kGemvWgsPerCu)), dim3(kGBlock), lds_d, L.s, cm, l,
                       xin0, (const float *)x->attn_norm[l], (const WT *)x->wqkv[l], q);
    L.after();
    const dim3 agrid(c.n_kv_heads, x->lay.n_splits, B);
    L.before(kKAttn);
#define ATTNB(HD, GG) hipLaunchKernelGGL((k_attn_b<WT, HD, GG>), agrid, dim3(kGBlock), 0, L.s, cm, l, (const float *)q, a, part, cnt)
    if (c.head_dim == 64) { if (G == 1) ATTNB(64, 1); else if (G == 2) ATTNB(64, 2); else ATTNB(64, 4); }
    else { if (G == 1) ATTNB(128, 1); else if (G == 2) ATTNB(128, 2); else ATTNB(128, 4); }
#undef ATTNB
    L.after();
    launch_proj_b<WT, B>(L, kKOproj, a, nq, (const WT *)x->wo[l], xin0, kXBatchWorkSlot0);
    L.before(kKGateUp);
    hipLaunchKernelGGL((k_gate_up_b<WT, B>), dim3(batch_grid(x, f, lds_d, kGateUpWgsPerCu)), dim3(kGBlock), lds_d, L.s, cm,
                       kXBatchWorkSlot0, (const float *)x->mlp_norm[l], (const WT *)x->wgu[l], mb);
    L.after();
    launch_proj_b<WT, B>(L, kKDown, mb, f, (const WT *)x->wdown[l], kXBatchWorkSlot0, kXBatchWorkSlot0);
  }
  float *logits = c.debug_logits > 0 ? at<float>(x, x->lay.logits) : nullptr;
  float *full = c.temperature > 0.0f ? at<float>(x, x->lay.logits_b) : nullptr;
  L.before(kKHead);
  hipLaunchKernelGGL((k_head_b<WT, B>), dim3(cm.dm.head_blocks), dim3(kGBlock), lds_d, L.s, cm, kXBatchWorkSlot0,
                     (const float *)x->final_norm, (const WT *)x->lm_head, sc<float2>(x, x->lay.cand_b), logits, full);
  L.after();
}

// Largest dynamic LDS the batched kernels of this B may be launched with.
template <typename WT, int B>
hipError_t allow_batch_lds() {
  const int bytes = (int)kBatchLdsMax;
  hipError_t e = hipFuncSetAttribute((const void *)k_qkv_b<WT, B>, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e == hipSuccess) e = hipFuncSetAttribute((const void *)k_gate_up_b<WT, B>, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e == hipSuccess) e = hipFuncSetAttribute((const void *)k_head_b<WT, B>, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e == hipSuccess) e = hipFuncSetAttribute((const void *)k_proj_resid_b<WT, B>, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e == hipSuccess) e = hipFuncSetAttribute((const void *)k_proj_resid_bs<WT, B>, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  return e;
}

template <typename WT>
hipError_t enqueue_eesd_round(ppsd_ctx *x) {
  const ppsd_config &c = x->cfg;
  Launcher A{x, x->sA, false};
  const int g = x->gamma;
  // gamma draft steps (layers 1..E + exit head on one token each), then the layer-E hidden state of
  // the last draft, each left in its batch slot
  for (int j = 0; j <= g; ++j) {
    launch_stage<WT>(A, kEesdDraft0 + j, 0, c.exit_layer, 0, kXStageWork0, true, kXBatchIn0 + j, kXStageWork0);
    if (c.exit_block) launch_exit_block<WT>(A, kEesdDraft0 + j, 0, kXBatchIn0 + j, kXStageWork0, j == g);
    if (j < g) {
      launch_head<WT>(A, kEesdDraft0 + j, c.exit_block ? kXStageWork0 : kXBatchIn0 + j, false);
      A.before(kKCommit);
      if (c.temperature > 0.0f)
        hipLaunchKernelGGL(k_eesd_pick_sample, dim3(1), dim3(kSBlock), 0, A.s, x->cm, at<const float>(x, x->lay.logits_exit),
                           at<float>(x, x->lay.probs_e), j, 1.0f / c.temperature, (uint32_t)c.sample_seed);
      else
        hipLaunchKernelGGL(k_eesd_pick, dim3(1), dim3(kBlock), 0, A.s, x->cm, sc<const float2>(x, x->lay.cand_exit), j);
      A.after();
    }
  }
  switch (g + 1) {
    case 2: launch_verify_batch<WT, 2>(A); break;
    case 3: launch_verify_batch<WT, 3>(A); break;
    case 4: launch_verify_batch<WT, 4>(A); break;
    default: launch_verify_batch<WT, 5>(A); break;
  }
  A.before(kKCommit);
  if (c.temperature > 0.0f)
    hipLaunchKernelGGL(k_eesd_commit_sample, dim3(1), dim3(kSBlock), 0, A.s, x->cm, at<const float>(x, x->lay.logits_b),
                       at<const float>(x, x->lay.probs_e), at<int32_t>(x, x->lay.out_tokens), at<int32_t>(x, x->lay.drafts), g,
                       1.0f / c.temperature, (uint32_t)c.sample_seed);
  else
    hipLaunchKernelGGL(k_eesd_commit, dim3(1), dim3(kBlock), 0, A.s, x->cm, sc<const float2>(x, x->lay.cand_b),
                       at<int32_t>(x, x->lay.out_tokens), at<int32_t>(x, x->lay.drafts), g);
  A.after();
  return A.err;
}

// One decode step in the given mode.  With two_streams the verify stage goes to stream B between
// a fork event and a join event (also valid under stream capture).
template <typename WT>
hipError_t enqueue_step(ppsd_ctx *x, int mode, bool two_streams, bool timed) {
  const ppsd_config &c = x->cfg;
  if (mode == PPSD_MODE_EESD) return enqueue_eesd_round<WT>(x);
  Launcher A{x, x->sA, timed};
  if (mode == PPSD_MODE_VANILLA) {
    launch_stage<WT>(A, kVanilla, 0, c.n_layers, 0, kXDraft, true, kXDraft);
    launch_head<WT>(A, kVanilla, kXDraft, true);
    launch_commit(A, 0);
    return A.err;
  }
  if (mode == PPSD_MODE_PIPELINE) {
    // One tick of the ceil(N/E)-stage schedule: every stage works on its own token, so the stages
    // are independent within a tick.  Stage k goes to stream k mod n_streams; a stream's stages run
    // one after the other and share that stream's scratch vectors.  Stage k reads the readable
    // buffer of boundary k and writes the other buffer of boundary k+1; the commit kernel swaps
    // the buffers when the tokens move on.
    const int S = x->cm.dm.n_stages;
    const int ns = two_streams ? x->n_streams : 1;
    hipError_t e = ns > 1 ? hipEventRecord(x->ev_fork, x->sA) : hipSuccess;
    for (int i = 1; i < ns && e == hipSuccess; ++i) e = hipStreamWaitEvent(x->sx[i], x->ev_fork, 0);
    if (e != hipSuccess) return e;
    for (int k = 0; k < S; ++k) {
      const int si = k % ns;
      Launcher Lk{x, x->sx[si], false};
      const int wl = later_stage_layers(&c);
      const int lo = k == 0 ? 0 : c.exit_layer + (k - 1) * wl;
      const int hi = k == 0 ? c.exit_layer : (lo + wl < c.n_layers ? lo + wl : c.n_layers);
      const int work = kXStageWork0 + k;
      const int xin = k == 0 ? work : kXBoundRead0 + k;
      const int xout = k == S - 1 ? work : kXBoundWrite0 + k + 1;
      launch_stage<WT>(Lk, kPipeStage0 + k, lo, hi, si, xin, k == 0, xout, work);
      if (k == 0 && c.exit_block) launch_exit_block<WT>(Lk, kPipeStage0, si, kXBoundWrite0 + 1, work, false);
      if (k == 0) launch_head<WT>(Lk, kPipeStage0, c.exit_block ? work : kXBoundWrite0 + 1, false);
      if (k == S - 1) launch_head<WT>(Lk, kPipeStage0 + k, work, true);
      if (Lk.err != hipSuccess) return Lk.err;
    }
    for (int i = 1; i < ns; ++i) {
      e = hipEventRecord(x->ev_joinx[i], x->sx[i]);
      if (e != hipSuccess) return e;
      e = hipStreamWaitEvent(x->sA, x->ev_joinx[i], 0);
      if (e != hipSuccess) return e;
    }
    launch_commit(A, 4);
    return A.err;
  }
  Launcher B{x, two_streams ? x->sB : x->sA, timed};
  if (two_streams) {
    hipError_t e = hipEventRecord(x->ev_fork, x->sA);
    if (e != hipSuccess) return e;
    e = hipStreamWaitEvent(x->sB, x->ev_fork, 0);
    if (e != hipSuccess) return e;
  }
  // draft stage: layers 1..E + exit head; its last layer writes the other hExit buffer
  launch_stage<WT>(A, kDraft, 0, c.exit_layer, 0, kXDraft, true, kHExitNext);
  if (c.exit_block) launch_exit_block<WT>(A, kDraft, 0, kHExitNext, kXDraft, false);
  launch_head<WT>(A, kDraft, c.exit_block ? kXDraft : kHExitNext, false);
  // verify stage: layers E+1..N + LM head on the hidden state kept from the previous step
  launch_stage<WT>(B, kVerify, c.exit_layer, c.n_layers, 1, kHExitCur, false, kXVerify);
  launch_head<WT>(B, kVerify, kXVerify, true);
  if (B.err != hipSuccess) return B.err;
  if (two_streams) {
    hipError_t e = hipEventRecord(x->ev_join, x->sB);
    if (e != hipSuccess) return e;
    e = hipStreamWaitEvent(x->sA, x->ev_join, 0);
    if (e != hipSuccess) return e;
  }
  launch_commit(A, 1);
  return A.err;
}

template <typename WT>
hipError_t enqueue_prefill_pos(ppsd_ctx *x, bool last, bool timed) {
  Launcher A{x, x->sA, timed};
  if (x->cfg.exit_block) {
    launch_stage<WT>(A, kPrefill, 0, x->cfg.exit_layer, 0, kXDraft, true, kXDraft);
    launch_exit_block<WT>(A, kPrefill, 0, kXDraft, kXDraft, true);
    launch_stage<WT>(A, kPrefill, x->cfg.exit_layer, x->cfg.n_layers, 0, kXDraft, false, kXDraft);
  } else {
    launch_stage<WT>(A, kPrefill, 0, x->cfg.n_layers, 0, kXDraft, true, kXDraft);
  }
  if (last) launch_head<WT>(A, kPrefill, kXDraft, true);
  launch_commit(A, last ? 3 : 2);
  return A.err;
}

hipError_t enqueue_step_any(ppsd_ctx *x, int mode, bool two_streams, bool timed) {
  return x->cfg.dtype == PPSD_FP32 ? enqueue_step<float>(x, mode, two_streams, timed)
                                   : enqueue_step<bf16_t>(x, mode, two_streams, timed);
}
hipError_t enqueue_prefill_any(ppsd_ctx *x, bool last, bool timed) {
  return x->cfg.dtype == PPSD_FP32 ? enqueue_prefill_pos<float>(x, last, timed)
                                   : enqueue_prefill_pos<bf16_t>(x, last, timed);
}

template <typename F>
int capture(ppsd_ctx *x, hipGraphExec_t *out, F &&body) {
  hipGraph_t g = nullptr;
  HIP_TRY(hipStreamBeginCapture(x->sA, hipStreamCaptureModeRelaxed));
  hipError_t e = body();
  hipError_t e2 = hipStreamEndCapture(x->sA, &g);
  if (e != hipSuccess) { if (g) (void)hipGraphDestroy(g); return fail(PPSD_EHIP, "capture body: %s", hipGetErrorString(e)); }
  if (e2 != hipSuccess) return fail(PPSD_EHIP, "hipStreamEndCapture: %s", hipGetErrorString(e2));
  hipError_t e3 = hipGraphInstantiate(out, g, nullptr, nullptr, 0);
  (void)hipGraphDestroy(g);
  if (e3 != hipSuccess) return fail(PPSD_EHIP, "hipGraphInstantiate: %s", hipGetErrorString(e3));
  return PPSD_OK;
}

// Drains the events recorded in profiling mode into the per-kind totals.  A launch whose
// stage was idle lasts a few microseconds and would distort the averages; those are skipped by
// the caller passing which kinds were active (all launches in serial profiling steps are
// counted only if the step's stage ran, see decode loop).
int drain_kernel_events(ppsd_ctx *x, const std::vector<char> *active_mask) {
  for (size_t k = 0; k + 1 < x->tk_used; ++k) {
    float ms = 0.f;
    HIP_TRY(hipEventElapsedTime(&ms, x->tk_events[k], x->tk_events[k + 1]));
    if (active_mask && !(*active_mask)[k]) continue;
    const int kind = x->tk_kinds[k];
    x->ktimes.total_us[kind] += 1000.0 * ms;
    x->ktimes.launches[kind] += 1;
  }
  x->tk_used = 0;
  return PPSD_OK;
}

// ---------------------------------------------------------------- persistent engine
MegaArgs mega_args(ppsd_ctx *x, bool prefill, int max_steps) {
  const ppsd_config &c = x->cfg;
  MegaArgs A{};
  A.cm = x->cm;
  A.layers = at<const LayerPtrs>(x, x->lay.layer_ptrs);
  A.embed = x->embed; A.final_norm = (const float *)x->final_norm; A.lm_head = x->lm_head;
  A.exit_norm = (const float *)x->exit_norm; A.exit_head = x->exit_head;
  for (int s = 0; s < 2; ++s) {
    A.q[s] = sc<float>(x, x->lay.q[s]); A.a[s] = sc<float>(x, x->lay.a[s]); A.m[s] = sc<float>(x, x->lay.mbuf[s]);
    A.partials[s] = sc<float>(x, x->lay.partials[s]); A.counters[s] = sc<int>(x, x->lay.counters[s]);
  }
  A.cand_lm = sc<float2>(x, x->lay.cand_lm); A.cand_exit = sc<float2>(x, x->lay.cand_exit);
  A.logits = c.debug_logits > 0 ? at<float>(x, x->lay.logits) : nullptr;
  A.out_tokens = at<int32_t>(x, x->lay.out_tokens); A.drafts = at<int32_t>(x, x->lay.drafts);
  A.cand_counts = at<int>(x, x->lay.cand_counts);
  A.bar = at<unsigned>(x, x->lay.bar); A.abort_flag = at<int>(x, x->lay.abort_flag);
  A.max_steps = max_steps; A.attn_splits = x->lay.n_splits; A.xs_stride = x->xs_stride;
  A.trace = (!prefill && x->trace_step >= 0) ? at<unsigned long long>(x, x->lay.trace) : nullptr;
  A.trace_step = x->trace_step; A.trace_wg = x->trace_wg;
  auto whole = [&](int role, int head) {
    return StageDesc{role, 0, c.n_layers, 0, kXDraft, 1, kXDraft, kXDraft, head, kXDraft};
  };
  if (prefill) {
    A.n_stages = 1; A.zip = 0; A.commit_kind = 2; A.st[0] = whole(kPrefill, 3);
  } else if (c.mode == PPSD_MODE_VANILLA) {
    A.n_stages = 1; A.zip = 0; A.commit_kind = 0; A.st[0] = whole(kVanilla, 1);
  } else {
    A.n_stages = 2; A.zip = c.mode == PPSD_MODE_OVERLAP ? 1 : 0; A.commit_kind = 1;
    A.st[0] = StageDesc{kDraft, 0, c.exit_layer, 0, kXDraft, 1, kXDraft, kHExitNext, 2, kHExitNext};
    A.st[1] = StageDesc{kVerify, c.exit_layer, c.n_layers, 1, kHExitCur, 0, kXVerify, kXVerify, 1, kXVerify};
  }
  return A;
}

template <typename WT>
const void *mega_fn_for(int hd, int g) {
  if (hd == 64) return g == 1 ? (const void *)k_mega<WT, 64, 1> : g == 2 ? (const void *)k_mega<WT, 64, 2> : (const void *)k_mega<WT, 64, 4>;
  return g == 1 ? (const void *)k_mega<WT, 128, 1> : g == 2 ? (const void *)k_mega<WT, 128, 2> : (const void *)k_mega<WT, 128, 4>;
}

const void *mega_fn(const ppsd_config &c) {
  const int g = c.n_heads / c.n_kv_heads;
  return c.dtype == PPSD_FP32 ? mega_fn_for<float>(c.head_dim, g) : mega_fn_for<bf16_t>(c.head_dim, g);
}

int mega_launch(ppsd_ctx *x, bool prefill, int max_steps) {
  MegaArgs A = mega_args(x, prefill, max_steps);
  HIP_TRY(hipMemsetAsync(A.bar, 0, 4, x->sA));
  HIP_TRY(hipMemsetAsync(A.abort_flag, 0, 4, x->sA));
  void *params[] = {&A};
  const void *fn = mega_fn(x->cfg);
  HIP_TRY(hipLaunchCooperativeKernel(fn, dim3(x->n_wg), dim3(kMBlock), params, (unsigned)x->mega_lds, x->sA));
  return PPSD_OK;
}

int mega_check_abort(ppsd_ctx *x) {
  int flag = 0;
  HIP_TRY(hipMemcpyAsync(&flag, at<int>(x, x->lay.abort_flag), 4, hipMemcpyDeviceToHost, x->sA));
  HIP_TRY(hipStreamSynchronize(x->sA));
  if (flag) return fail(PPSD_EHIP, "persistent kernel gave up at a grid barrier (bounded wait expired)");
  return PPSD_OK;
}

int mega_setup(ppsd_ctx *x) {
  const ppsd_config &c = x->cfg;
  int dev = 0;
  HIP_TRY(hipGetDevice(&dev));
  hipDeviceProp_t prop;
  HIP_TRY(hipGetDeviceProperties(&prop, dev));
  if (!prop.cooperativeLaunch) return fail(PPSD_EARG, "device does not support cooperative launches");
  if (c.d_model > 16 * kMBlock) return fail(PPSD_EARG, "persistent engine supports d_model <= %d", 16 * kMBlock);
  const int nq = c.n_heads * c.head_dim;
  int xs = c.d_model > nq ? c.d_model : nq;
  if (c.d_ffn > xs) xs = c.d_ffn;
  x->xs_stride = xs_floats(c.dtype == PPSD_FP32 ? 4 : 2, xs);
  const int vec = c.dtype == PPSD_FP32 ? 4 : 8;
  const int G = c.n_heads / c.n_kv_heads;
  const size_t merge_floats = (size_t)(kMBlock / (c.head_dim / vec)) * G * (c.head_dim + 2);
  size_t lds_floats = (size_t)x->xs_stride;          // one staged input vector per workgroup
  if (merge_floats > lds_floats) lds_floats = merge_floats;
  x->mega_lds = lds_floats * 4;
  const void *fn = mega_fn(c);
  HIP_TRY(hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)x->mega_lds));
  int per_cu = 0;
  HIP_TRY(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, kMBlock, x->mega_lds));
  if (per_cu < 1) return fail(PPSD_EARG, "persistent kernel does not fit on a CU (LDS %zu bytes)", x->mega_lds);
  if (per_cu > kMegaWgsPerCu) per_cu = kMegaWgsPerCu;
  x->n_wg = per_cu * x->n_cu;
  if (x->n_wg > kMaxWorkgroups) x->n_wg = kMaxWorkgroups;
  std::vector<LayerPtrs> lp(c.n_layers);
  for (int l = 0; l < c.n_layers; ++l)
    lp[l] = LayerPtrs{(const float *)x->attn_norm[l], x->wqkv[l], x->wo[l], (const float *)x->mlp_norm[l], x->wgu[l], x->wdown[l]};
  HIP_TRY(hipMemcpyAsync(at<LayerPtrs>(x, x->lay.layer_ptrs), lp.data(), sizeof(LayerPtrs) * lp.size(), hipMemcpyHostToDevice, x->sA));
  HIP_TRY(hipStreamSynchronize(x->sA));
  return PPSD_OK;
}

// ---------------------------------------------------------------- matrix-core prefill
template <int EPI>
void pf_launch_gemm(ppsd_ctx *x, PfGemm g, int n_cols) {
  g.part = at<float>(x, x->lay.pf_part);
  pf_launch<EPI>(x->sA, x->cm, g, pf_plan(g.n_valid, n_cols, g.K, x->cfg.tune_prefill_tile ? x->cfg.tune_prefill_tile : -1));
}

// Attention of a chunk's queries (group sizes 1, 2, 4: what valid_config admits).
void pf_launch_attn(ppsd_ctx *x, int l, int c0, int nv, const float *Q, float *AO) {
  const ppsd_config &c = x->cfg;
  const int G = c.n_heads / c.n_kv_heads, qp = kPfBM / G;
  const dim3 grid(c.n_kv_heads, (nv + qp - 1) / qp);
  if (G == 1) hipLaunchKernelGGL((k_pf_flash<1>), grid, dim3(kPfBlock), 0, x->sA, x->cm, l, c0, nv, Q, AO);
  else if (G == 2) hipLaunchKernelGGL((k_pf_flash<2>), grid, dim3(kPfBlock), 0, x->sA, x->cm, l, c0, nv, Q, AO);
  else hipLaunchKernelGGL((k_pf_flash<4>), grid, dim3(kPfBlock), 0, x->sA, x->cm, l, c0, nv, Q, AO);
}

int prefill_mfma(ppsd_ctx *x, int n_prompt) {
  const ppsd_config &c = x->cfg;
  if (c.dtype != PPSD_BF16) return fail(PPSD_ESTATE, "matrix-core prefill is bf16 only");
  const int d = c.d_model, f = c.d_ffn, nq = c.n_heads * c.head_dim;
  const int qkv_cols = (c.n_heads + 2 * c.n_kv_heads) * c.head_dim, G = c.n_heads / c.n_kv_heads;
  float *X = at<float>(x, x->lay.pf_x), *Q = at<float>(x, x->lay.pf_q), *AO = at<float>(x, x->lay.pf_ao);
  bf16_t *Ah = at<bf16_t>(x, x->lay.pf_ah), *Al = at<bf16_t>(x, x->lay.pf_al);
  bf16_t *Mh = at<bf16_t>(x, x->lay.pf_mh), *Ml = at<bf16_t>(x, x->lay.pf_ml);
  const int waves = kPfBlock / kWave, chunk = x->lay.pf_chunk;
  for (int c0 = 0; c0 < n_prompt; c0 += chunk) {
    const int nv = n_prompt - c0 < chunk ? n_prompt - c0 : chunk;
    const dim3 sgrid((nv + waves - 1) / waves);
    hipLaunchKernelGGL(k_pf_embed, dim3(nv), dim3(kPfBlock), 0, x->sA, (const bf16_t *)x->embed, x->cm.prompt, c0, nv, d, X);
    for (int l = 0; l < c.n_layers; ++l) {
      PfGemm g{};
      g.n_valid = nv; g.c0 = c0; g.layer = l; g.X = X; g.Q = Q; g.Mh = Mh; g.Ml = Ml; g.Ah = Ah; g.Al = Al;
      hipLaunchKernelGGL(k_pf_split, sgrid, dim3(kPfBlock), 0, x->sA, (const float *)X, d, nv, (const float *)x->attn_norm[l], c.rms_eps, Ah, Al);
      g.W = (const bf16_t *)x->wqkv[l]; g.K = d;
      pf_launch_gemm<kPfQkv>(x, g, qkv_cols);
      pf_launch_attn(x, l, c0, nv, Q, AO);
      hipLaunchKernelGGL(k_pf_split, sgrid, dim3(kPfBlock), 0, x->sA, (const float *)AO, nq, nv, (const float *)nullptr, 0.0f, Ah, Al);
      g.W = (const bf16_t *)x->wo[l]; g.K = nq;
      pf_launch_gemm<kPfResid>(x, g, d);
      hipLaunchKernelGGL(k_pf_split, sgrid, dim3(kPfBlock), 0, x->sA, (const float *)X, d, nv, (const float *)x->mlp_norm[l], c.rms_eps, Ah, Al);
      g.W = (const bf16_t *)x->wgu[l]; g.K = d;
      pf_launch_gemm<kPfSwiglu>(x, g, 2 * f);
      g.Ah = Mh; g.Al = Ml; g.W = (const bf16_t *)x->wdown[l]; g.K = f;
      pf_launch_gemm<kPfResid>(x, g, d);
      if (c.exit_block && l == c.exit_layer - 1) {
        // K/V rows of the early-exit block for the prompt positions: its QKV projection on h^E
        // (the q it also writes is overwritten by the next layer)
        const int xl = c.n_layers;
        hipLaunchKernelGGL(k_pf_split, sgrid, dim3(kPfBlock), 0, x->sA, (const float *)X, d, nv, (const float *)x->attn_norm[xl], c.rms_eps, Ah, Al);
        g.layer = xl; g.Ah = Ah; g.Al = Al; g.W = (const bf16_t *)x->wqkv[xl]; g.K = d;
        pf_launch_gemm<kPfQkv>(x, g, qkv_cols);
      }
      HIP_TRY(hipGetLastError());
    }
    if (c0 + nv == n_prompt)
      hipLaunchKernelGGL(k_pf_last_row, dim3(4), dim3(256), 0, x->sA, (const float *)X, nv - 1, d, x->cm.xbuf + (size_t)kXDraft * d);
  }
  // the LM head and the commit run as for the last position of the looped prefill
  hipLaunchKernelGGL(k_begin_prefill, dim3(1), dim3(64), 0, x->sA, at<DevState>(x, x->lay.state), n_prompt, n_prompt - 1);
  Launcher A{x, x->sA, false};
  launch_head<bf16_t>(A, kPrefill, kXDraft, true);
  launch_commit(A, 3);
  if (A.err != hipSuccess) return fail(PPSD_EHIP, "prefill head: %s", hipGetErrorString(A.err));
  HIP_TRY(hipGetLastError());
  return PPSD_OK;
}

int read_state(ppsd_ctx *x) {
  HIP_TRY(hipMemcpyAsync(x->h_state, at<DevState>(x, x->lay.state), sizeof(DevState), hipMemcpyDeviceToHost, x->sA));
  HIP_TRY(hipStreamSynchronize(x->sA));
  return PPSD_OK;
}

}  // namespace

extern "C" {

const char *ppsd_last_error(void) { return g_err.c_str(); }

size_t ppsd_workspace_bytes(const ppsd_config *cfg) {
  const char *why = "";
  if (!valid_config(cfg, &why)) { fail(PPSD_EARG, "invalid config: %s", why); return 0; }
  return make_layout(cfg).total;
}

int ppsd_load_weights(const ppsd_config *cfg, const ppsd_buffers *b, ppsd_ctx **out) {
  const char *why = "";
  if (!out) return fail(PPSD_EARG, "out is null");
  *out = nullptr;
  if (!valid_config(cfg, &why)) return fail(PPSD_EARG, "invalid config: %s", why);
  if (!b) return fail(PPSD_EARG, "buffers is null");
  if (!b->embed || !b->final_norm || !b->lm_head || !b->exit_norm || !b->exit_head || !b->attn_norm || !b->wqkv ||
      !b->wo || !b->mlp_norm || !b->wgu || !b->wdown || !b->workspace)
    return fail(PPSD_EARG, "a weight or workspace pointer is null");
  if (!b->stream_draft || !b->stream_verify || b->stream_draft == b->stream_verify)
    return fail(PPSD_EARG, "two distinct non-default streams are required");
  const Layout lay = make_layout(cfg);
  if (b->workspace_bytes < lay.total)
    return fail(PPSD_ECAPACITY, "workspace has %zu bytes, %zu needed", b->workspace_bytes, lay.total);
  if ((uintptr_t)b->workspace % kAlign) return fail(PPSD_EARG, "workspace must be 256-byte aligned");
  for (int l = 0; l < cfg->n_layers + cfg->exit_block; ++l) {
    const void *ps[6] = {b->attn_norm[l], b->wqkv[l], b->wo[l], b->mlp_norm[l], b->wgu[l], b->wdown[l]};
    for (const void *p : ps) {
      if (!p) return fail(PPSD_EARG, "layer %d has a null weight pointer", l);
      if ((uintptr_t)p % 16) return fail(PPSD_EARG, "layer %d has a weight pointer that is not 16-byte aligned", l);
    }
  }
  const void *gl[5] = {b->embed, b->final_norm, b->lm_head, b->exit_norm, b->exit_head};
  for (const void *p : gl)
    if ((uintptr_t)p % 16) return fail(PPSD_EARG, "a global weight pointer is not 16-byte aligned");
  std::vector<int32_t> table(lay.n_pages);
  {
    std::vector<char> seen(lay.n_pages, 0);
    for (int p = 0; p < lay.n_pages; ++p) {
      const int32_t v = b->kv_page_table ? b->kv_page_table[p] : p;
      if (v < 0 || v >= lay.n_pages || seen[v]) return fail(PPSD_EARG, "kv_page_table is not a permutation");
      seen[v] = 1;
      table[p] = v;
    }
  }

  ppsd_ctx *x = new (std::nothrow) ppsd_ctx();
  if (!x) return fail(PPSD_EARG, "out of host memory");
  x->cfg = *cfg;
  x->lay = lay;
  x->ws = (char *)b->workspace;
  x->scr = x->ws + lay.scratch0;
  x->embed = b->embed; x->final_norm = b->final_norm; x->lm_head = b->lm_head;
  x->exit_norm = b->exit_norm; x->exit_head = b->exit_head;
  x->attn_norm.assign(b->attn_norm, b->attn_norm + cfg->n_layers + cfg->exit_block);
  x->wqkv.assign(b->wqkv, b->wqkv + cfg->n_layers + cfg->exit_block);
  x->wo.assign(b->wo, b->wo + cfg->n_layers + cfg->exit_block);
  x->mlp_norm.assign(b->mlp_norm, b->mlp_norm + cfg->n_layers + cfg->exit_block);
  x->wgu.assign(b->wgu, b->wgu + cfg->n_layers + cfg->exit_block);
  x->wdown.assign(b->wdown, b->wdown + cfg->n_layers + cfg->exit_block);
  x->sA = (hipStream_t)b->stream_draft;
  x->sB = (hipStream_t)b->stream_verify;

  Common &cm = x->cm;
  cm.st = at<DevState>(x, lay.state);
  cm.prompt = at<int32_t>(x, lay.prompt);
  cm.xbuf = at<float>(x, lay.xbuf);
  cm.rope_cos = at<float>(x, lay.rope_cos);
  cm.rope_sin = at<float>(x, lay.rope_sin);
  cm.page_table = at<int32_t>(x, lay.page_table);
  cm.kv_pool = x->ws + lay.kv;
  Dims &m = cm.dm;
  m.d = cfg->d_model; m.n_h = cfg->n_heads; m.n_kv = cfg->n_kv_heads; m.hd = cfg->head_dim; m.f = cfg->d_ffn;
  m.V = cfg->vocab; m.L = cfg->n_layers; m.E = cfg->exit_layer; m.max_seq = cfg->max_seq;
  m.page_tokens = cfg->kv_page_tokens; m.n_pages = lay.n_pages; m.n_splits = lay.n_splits;
  m.debug_rows = cfg->debug_logits; m.head_blocks = 0;   // set below, once the device is known
  m.n_stages = pipeline_stages(cfg);
  m.page_shift = 0;
  while ((1 << m.page_shift) < cfg->kv_page_tokens) ++m.page_shift;
  m.eps = cfg->rms_eps; m.qscale = (float)(1.0 / std::sqrt((double)cfg->head_dim));
  {
    // default: the draft stage's bytes over the verify stage's (7B, E = 8 of 32: 0.35; measured on the 7B and
    // 13B workloads, shares of 25-40 % give 2-3 % more tokens/s than equal grids, 17 % loses again)
    const double layer = (double)(cfg->n_heads + 2 * cfg->n_kv_heads) * cfg->head_dim * cfg->d_model +
                         (double)cfg->d_model * cfg->n_heads * cfg->head_dim + 3.0 * cfg->d_ffn * cfg->d_model;
    const double head = (double)cfg->vocab * cfg->d_model;
    const double ratio = ((cfg->exit_layer + cfg->exit_block) * layer + head) / ((cfg->n_layers - cfg->exit_layer) * layer + head);
    int share = (int)(256.0 * ratio + 0.5);
    share = share < 32 ? 32 : share > 256 ? 256 : share;
    m.draft_share = cfg->tune_draft_share ? (cfg->tune_draft_share * 256 + 50) / 100 : share;
    if (cfg->mode != PPSD_MODE_OVERLAP || cfg->time_kernels) m.draft_share = 256;   // only there do the two stages run side by side
  }

  auto cleanup = [&](int rc) { ppsd_free(x); return rc; };
  {
    int dev = 0, n_cu = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n_cu < 1)
      return cleanup(fail(PPSD_EHIP, "cannot query the device's compute-unit count"));
    x->n_cu = n_cu;
    m.head_blocks = x->gemv_grid((cfg->vocab + 1) / 2);
    if (cfg->tune_attn_split == 0 && cfg->max_seq > kOneSplitUpTo) {
      // long contexts: as many splits as fill the chip (one attention workgroup is resident per compute
      // unit), a block of 128 positions per split at least
      int fill = n_cu / cfg->n_kv_heads;
      if (fill > cfg->max_seq / 128) fill = cfg->max_seq / 128;
      if (fill > kMaxSplits) fill = kMaxSplits;
      if (fill > x->lay.n_splits) { x->lay.n_splits = fill; m.n_splits = fill; }
    }
  }
#define HIP_TRY_X(expr)                                                                                   \
  do {                                                                                                    \
    hipError_t e_ = (expr);                                                                               \
    if (e_ != hipSuccess) return cleanup(fail(PPSD_EHIP, "%s: %s", #expr, hipGetErrorString(e_)));        \
  } while (0)
  HIP_TRY_X(hipEventCreateWithFlags(&x->ev_fork, hipEventDisableTiming));
  HIP_TRY_X(hipEventCreateWithFlags(&x->ev_join, hipEventDisableTiming));
  x->sx[0] = x->sA; x->sx[1] = x->sB;
  if (x->lay.pf) HIP_TRY_X(pf_prepare());
  if (cfg->mode == PPSD_MODE_EESD) {
    x->gamma = cfg->eesd_gamma ? cfg->eesd_gamma : kDefaultGamma;
    hipError_t e = hipSuccess;
    const bool f32 = cfg->dtype == PPSD_FP32;
    switch (x->gamma + 1) {
      case 2: e = f32 ? allow_batch_lds<float, 2>() : allow_batch_lds<bf16_t, 2>(); break;
      case 3: e = f32 ? allow_batch_lds<float, 3>() : allow_batch_lds<bf16_t, 3>(); break;
      case 4: e = f32 ? allow_batch_lds<float, 4>() : allow_batch_lds<bf16_t, 4>(); break;
      default: e = f32 ? allow_batch_lds<float, 5>() : allow_batch_lds<bf16_t, 5>(); break;
    }
    HIP_TRY_X(e);
  }
  if (cfg->mode == PPSD_MODE_PIPELINE) {
    const int S = m.n_stages;
    x->n_streams = cfg->pipeline_streams ? cfg->pipeline_streams : (S < kMaxStreams ? S : kMaxStreams);
    if (x->n_streams > S) x->n_streams = S;
    for (int i = 2; i < x->n_streams; ++i) HIP_TRY_X(hipStreamCreateWithFlags(&x->sx[i], hipStreamNonBlocking));
    for (int i = 1; i < x->n_streams; ++i) HIP_TRY_X(hipEventCreateWithFlags(&x->ev_joinx[i], hipEventDisableTiming));
  }
  HIP_TRY_X(hipEventCreate(&x->ev_t0));
  HIP_TRY_X(hipEventCreate(&x->ev_t1));
  HIP_TRY_X(hipHostMalloc((void **)&x->h_state, sizeof(DevState), hipHostMallocDefault));
  HIP_TRY_X(hipHostMalloc((void **)&x->h_out, 4ull * cfg->max_seq, hipHostMallocDefault));
  {
    int dev = 0;
    HIP_TRY_X(hipGetDevice(&dev));
    x->device = dev;
    if (dev >= 0 && dev < kMaxDevices && !g_static_scratch[dev]) {
      void *p = nullptr;
      HIP_TRY_X(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
      g_static_scratch[dev] = p;
    }
  }

  // everything before the KV pool starts from zero (state, counters, candidates, logs)
  HIP_TRY_X(hipMemsetAsync(x->ws, 0, lay.kv, x->sA));
  HIP_TRY_X(hipMemcpyAsync(at<int32_t>(x, lay.page_table), table.data(), 4ull * lay.n_pages, hipMemcpyHostToDevice, x->sA));
  {
    // rotary table in double on the host: angle = pos * base^(-2i/hd)
    const int half = cfg->head_dim / 2;
    std::vector<float> cs((size_t)cfg->max_seq * half), sn((size_t)cfg->max_seq * half);
    for (int i = 0; i < half; ++i) {
      const double theta = std::pow((double)cfg->rope_base, -2.0 * i / cfg->head_dim);
      for (int p = 0; p < cfg->max_seq; ++p) {
        const double ang = (double)p * theta;
        cs[(size_t)p * half + i] = (float)std::cos(ang);
        sn[(size_t)p * half + i] = (float)std::sin(ang);
      }
    }
    HIP_TRY_X(hipMemcpyAsync(at<float>(x, lay.rope_cos), cs.data(), cs.size() * 4, hipMemcpyHostToDevice, x->sA));
    HIP_TRY_X(hipMemcpyAsync(at<float>(x, lay.rope_sin), sn.data(), sn.size() * 4, hipMemcpyHostToDevice, x->sA));
    HIP_TRY_X(hipStreamSynchronize(x->sA));   // host vectors go out of scope
  }

  if (cfg->engine == PPSD_ENGINE_PERSISTENT) {
    int rc = mega_setup(x);
    if (rc != PPSD_OK) return cleanup(rc);
  } else if (cfg->use_graph && !cfg->time_kernels) {
    int rc = capture(x, &x->g_step, [&] { return enqueue_step_any(x, cfg->mode, cfg->mode == PPSD_MODE_OVERLAP || cfg->mode == PPSD_MODE_PIPELINE, false); });
    if (rc != PPSD_OK) return cleanup(rc);
    rc = capture(x, &x->g_prefill, [&] { return enqueue_prefill_any(x, false, false); });
    if (rc != PPSD_OK) return cleanup(rc);
  }
#undef HIP_TRY_X
  *out = x;
  return PPSD_OK;
}

void ppsd_free(ppsd_ctx *x) {
  if (!x) return;
  if (x->sA) (void)hipStreamSynchronize(x->sA);
  if (x->sB) (void)hipStreamSynchronize(x->sB);
  for (int i = 2; i < kMaxStreams; ++i) if (x->sx[i]) (void)hipStreamSynchronize(x->sx[i]);
  if (x->g_step) (void)hipGraphExecDestroy(x->g_step);
  if (x->g_prefill) (void)hipGraphExecDestroy(x->g_prefill);
  if (x->ev_fork) (void)hipEventDestroy(x->ev_fork);
  if (x->ev_join) (void)hipEventDestroy(x->ev_join);
  for (int i = 0; i < kMaxStreams; ++i) if (x->ev_joinx[i]) (void)hipEventDestroy(x->ev_joinx[i]);
  for (int i = 2; i < kMaxStreams; ++i) if (x->sx[i]) (void)hipStreamDestroy(x->sx[i]);
  if (x->ev_t0) (void)hipEventDestroy(x->ev_t0);
  if (x->ev_t1) (void)hipEventDestroy(x->ev_t1);
  for (hipEvent_t e : x->tk_events) (void)hipEventDestroy(e);
  if (x->h_state) (void)hipHostFree(x->h_state);
  if (x->h_out) (void)hipHostFree(x->h_out);
  delete x;
}

int ppsd_prefill(ppsd_ctx *x, const int32_t *prompt, int32_t n_prompt, int32_t *first_token) {
  if (!x || !prompt || !first_token) return fail(PPSD_EARG, "null argument");
  if (n_prompt < 1) return fail(PPSD_EARG, "n_prompt must be >= 1");
  if (n_prompt + 2 > x->cfg.max_seq)
    return fail(PPSD_ECAPACITY, "prompt of %d tokens does not fit max_seq %d", n_prompt, x->cfg.max_seq);
  for (int i = 0; i < n_prompt; ++i)
    if (prompt[i] < 0 || prompt[i] >= x->cfg.vocab) return fail(PPSD_EARG, "prompt[%d] = %d is outside the vocabulary", i, prompt[i]);
  x->prefilled = false;
  HIP_TRY(hipMemcpyAsync(at<int32_t>(x, x->lay.prompt), prompt, 4ull * n_prompt, hipMemcpyHostToDevice, x->sA));
  hipLaunchKernelGGL(k_begin_prefill, dim3(1), dim3(64), 0, x->sA, at<DevState>(x, x->lay.state), n_prompt, 0);
  HIP_TRY(hipGetLastError());
  int rc;
  if (x->lay.pf) {
    rc = prefill_mfma(x, n_prompt);
    if (rc != PPSD_OK) return rc;
  } else if (x->cfg.engine == PPSD_ENGINE_PERSISTENT) {
    rc = mega_launch(x, true, n_prompt);
    if (rc != PPSD_OK) return rc;
    rc = mega_check_abort(x);
    if (rc != PPSD_OK) return rc;
  } else {
    for (int p = 0; p < n_prompt; ++p) {
      const bool last = p == n_prompt - 1;
      if (!last && x->g_prefill) HIP_TRY(hipGraphLaunch(x->g_prefill, x->sA));
      else HIP_TRY(enqueue_prefill_any(x, last, false));
    }
  }
  rc = read_state(x);
  if (rc != PPSD_OK) return rc;
  if (x->h_state->prefill_pos != n_prompt || x->h_state->t != n_prompt)
    return fail(PPSD_ESTATE, "prefill ended in an unexpected device state (pos %d, t %d)", x->h_state->prefill_pos, x->h_state->t);
  *first_token = x->h_state->last_token;
  x->prefilled = true;
  x->host_len = n_prompt + 1;
  x->steps_launched = 0;
  x->device_ms = 0.0;
  x->ktimes = ppsd_kernel_times_t{};
  return PPSD_OK;
}

static int decode_impl(ppsd_ctx *x, int32_t n_tokens, int32_t *out_tokens, int32_t *n_written, bool static_scratch);

int ppsd_decode(ppsd_ctx *x, int32_t n_tokens, int32_t *out_tokens, int32_t *n_written) {
  return decode_impl(x, n_tokens, out_tokens, n_written, false);
}

int ppsd_decode_static_scratch(ppsd_ctx *x, int32_t n_tokens, int32_t *out_tokens, int32_t *n_written) {
  if (!x || !n_written) return fail(PPSD_EARG, "null argument");
  *n_written = 0;
  if (x->cfg.engine != PPSD_ENGINE_STREAMS || x->cfg.time_kernels)
    return fail(PPSD_EARG, "ppsd_decode_static_scratch runs on the per-operation engine, without time_kernels");
  if (x->lay.scratch_bytes > (size_t)PPSD_STATIC_SCRATCH_BYTES)
    return fail(PPSD_ECAPACITY, "this configuration needs %zu bytes of per-step scratch, the static region holds %zu",
                x->lay.scratch_bytes, (size_t)PPSD_STATIC_SCRATCH_BYTES);
  int dev = -1;
  HIP_TRY(hipGetDevice(&dev));
  if (dev != x->device || dev < 0 || dev >= kMaxDevices || !g_static_scratch[dev])
    return fail(PPSD_ESTATE, "the context was created on device %d, the current device is %d", x->device, dev);
  // The region keeps what the last call (of any context on this device) left.  The kernels write every
  // buffer before they read it, except the arrival counters of the attention splits, which must start at zero.
  char *const own = x->scr;
  x->scr = (char *)g_static_scratch[dev];
  const int n_ctr = kCounterStride * x->cfg.n_kv_heads;
  for (int s = 0; s < kMaxStreams; ++s)
    hipLaunchKernelGGL(k_fill_int, dim3((n_ctr + 255) / 256), dim3(256), 0, x->sA, sc<int>(x, x->lay.counters[s]), n_ctr, 0);
  if (x->cfg.mode == PPSD_MODE_EESD)
    hipLaunchKernelGGL(k_fill_int, dim3((kMaxBatch * n_ctr + 255) / 256), dim3(256), 0, x->sA, sc<int>(x, x->lay.counters_b),
                       kMaxBatch * n_ctr, 0);
  int rc = hipGetLastError() == hipSuccess ? PPSD_OK : fail(PPSD_EHIP, "clearing the static scratch counters failed");
  if (rc == PPSD_OK) rc = decode_impl(x, n_tokens, out_tokens, n_written, true);
  x->scr = own;
  return rc;
}

static int decode_impl(ppsd_ctx *x, int32_t n_tokens, int32_t *out_tokens, int32_t *n_written, bool static_scratch) {
  if (!x || !n_written || (n_tokens > 0 && !out_tokens)) return fail(PPSD_EARG, "null argument");
  *n_written = 0;
  if (n_tokens < 0) return fail(PPSD_EARG, "n_tokens < 0");
  if (!x->prefilled) return fail(PPSD_ESTATE, "ppsd_decode before ppsd_prefill");
  if (n_tokens == 0) return PPSD_OK;
  // positions 0..host_len-1 are committed; committing n more needs rows up to host_len+n-1 plus
  // the speculative rows written ahead of the last committed token: one by the draft stage, or
  // one per stage in front of the last one in the full pipeline schedule
  const int spec = x->cfg.mode == PPSD_MODE_PIPELINE ? x->cm.dm.n_stages - 1 : x->cfg.mode == PPSD_MODE_EESD ? x->gamma : 1;
  if ((int64_t)x->host_len + n_tokens + spec > x->cfg.max_seq)
    return fail(PPSD_ECAPACITY, "%d committed + %d new + %d speculative position(s) exceed max_seq %d", x->host_len, n_tokens,
                spec, x->cfg.max_seq);
  const ppsd_config &c = x->cfg;
  const bool timed = c.time_kernels != 0;
  const bool two = (c.mode == PPSD_MODE_OVERLAP || c.mode == PPSD_MODE_PIPELINE) && !timed;
  hipLaunchKernelGGL(k_begin_decode, dim3(1), dim3(64), 0, x->sA, at<DevState>(x, x->lay.state), n_tokens);
  HIP_TRY(hipGetLastError());
  HIP_TRY(hipEventRecord(x->ev_t0, x->sA));
  int remaining = n_tokens;
  int guard = 0;
  while (remaining > 0) {
    if (c.engine == PPSD_ENGINE_PERSISTENT) {
      // each step commits at most one token and at least every second step commits one
      const int max_steps = 2 * remaining + 2;
      int rc = mega_launch(x, false, max_steps);
      if (rc != PPSD_OK) return rc;
      x->steps_launched += 1;
      rc = mega_check_abort(x);
      if (rc != PPSD_OK) return rc;
      rc = read_state(x);
      if (rc != PPSD_OK) return rc;
    } else if (timed) {
      if (x->ktimes.event_overhead_us == 0.0) {
        // what an event adds between two launches: 64 empty kernels with an event after each, against
        // 64 empty kernels back to back
        Launcher cal{x, x->sA, true};
        const int n_cal = 64;
        cal.need_event(n_cal);
        if (cal.err != hipSuccess) return fail(PPSD_EHIP, "hipEventCreate: %s", hipGetErrorString(cal.err));
        float with_ev = 0.f, without = 0.f;
        for (int pass = 0; pass < 2; ++pass) {      // the first pass warms the kernel up
          HIP_TRY(hipStreamSynchronize(x->sA));
          HIP_TRY(hipEventRecord(x->tk_events[0], x->sA));
          for (int k = 1; k <= n_cal; ++k) {
            hipLaunchKernelGGL(k_nop, dim3(1), dim3(64), 0, x->sA, (int *)nullptr);
            HIP_TRY(hipEventRecord(x->tk_events[k], x->sA));
          }
          HIP_TRY(hipStreamSynchronize(x->sA));
          HIP_TRY(hipEventElapsedTime(&with_ev, x->tk_events[0], x->tk_events[n_cal]));
          HIP_TRY(hipEventRecord(x->tk_events[0], x->sA));
          for (int k = 1; k <= n_cal; ++k) hipLaunchKernelGGL(k_nop, dim3(1), dim3(64), 0, x->sA, (int *)nullptr);
          HIP_TRY(hipEventRecord(x->tk_events[1], x->sA));
          HIP_TRY(hipStreamSynchronize(x->sA));
          HIP_TRY(hipEventElapsedTime(&without, x->tk_events[0], x->tk_events[1]));
        }
        HIP_TRY(hipGetLastError());
        const double ev = 1000.0 * (with_ev - without) / n_cal;
        x->ktimes.event_overhead_us = ev > 1e-3 ? ev : 1e-3;
      }
      // one step at a time so idle launches can be told apart from active ones
      int rc = read_state(x);
      if (rc != PPSD_OK) return rc;
      const int was_full = x->h_state->full;
      HIP_TRY(enqueue_step_any(x, c.mode, false, true));
      x->steps_launched += 1;
      rc = read_state(x);
      if (rc != PPSD_OK) return rc;
      std::vector<char> mask(x->tk_used > 0 ? x->tk_used - 1 : 0, 1);
      if (c.mode != PPSD_MODE_VANILLA && !was_full) {
        // draft-only step: the verify stage's launches (after the draft stage's 5E+1) were idle
        const size_t draft_launches = 5u * c.exit_layer + 1;
        for (size_t k = draft_launches; k + 1 < mask.size(); ++k) mask[k] = 0;   // keep the commit
      }
      rc = drain_kernel_events(x, &mask);
      if (rc != PPSD_OK) return rc;
    } else {
      // a step commits at most one token; a draft-then-verify round at most gamma + 1
      const int per = c.mode == PPSD_MODE_EESD ? x->gamma + 1 : 1;
      const int n_steps = (remaining + per - 1) / per;
      for (int k = 0; k < n_steps; ++k) {
        // the captured graph holds the workspace's scratch addresses: the static-scratch variant launches directly
        if (x->g_step && !static_scratch) HIP_TRY(hipGraphLaunch(x->g_step, x->sA));
        else HIP_TRY(enqueue_step_any(x, c.mode, two, false));
      }
      x->steps_launched += n_steps;
      int rc = read_state(x);
      if (rc != PPSD_OK) return rc;
    }
    remaining = n_tokens - x->h_state->n_out;
    if (++guard > 4 * n_tokens + 16) return fail(PPSD_ESTATE, "decode made no progress (device state n_out %d)", x->h_state->n_out);
  }
  HIP_TRY(hipEventRecord(x->ev_t1, x->sA));
  // through the context's pinned block: a copy into pageable memory may make the runtime allocate staging
  HIP_TRY(hipMemcpyAsync(x->h_out, at<int32_t>(x, x->lay.out_tokens), 4ull * n_tokens, hipMemcpyDeviceToHost, x->sA));
  HIP_TRY(hipStreamSynchronize(x->sA));
  HIP_TRY(hipStreamSynchronize(x->sB));
  std::memcpy(out_tokens, x->h_out, 4ull * n_tokens);
  float ms = 0.f;
  HIP_TRY(hipEventElapsedTime(&ms, x->ev_t0, x->ev_t1));
  x->device_ms += ms;
  x->host_len += n_tokens;
  *n_written = n_tokens;
  return PPSD_OK;
}

int ppsd_stats(const ppsd_ctx *cx, ppsd_stats_t *out) {
  if (!cx || !out) return fail(PPSD_EARG, "null argument");
  ppsd_ctx *x = const_cast<ppsd_ctx *>(cx);
  int rc = read_state(x);
  if (rc != PPSD_OK) return rc;
  const int64_t *s = x->h_state->stats;
  out->committed = s[0]; out->drafts_compared = s[1]; out->accepted = s[2]; out->rejected = s[3];
  out->steps_overlapped = s[4]; out->steps_draft_only = s[5]; out->kv_rollbacks = s[6];
  out->steps_launched = x->steps_launched;
  out->device_ms = x->device_ms;
  out->pipeline_ticks = s[8]; out->stage_runs = s[9]; out->flushed_tokens = s[10]; out->eesd_rounds = s[11];
  return PPSD_OK;
}

int ppsd_read_logits(ppsd_ctx *x, int32_t first, int32_t count, float *out) {
  if (!x || !out) return fail(PPSD_EARG, "null argument");
  if (first < 0 || count < 0 || first + count > x->cfg.debug_logits)
    return fail(PPSD_EARG, "rows %d..%d are outside the %d kept logit rows", first, first + count - 1, x->cfg.debug_logits);
  HIP_TRY(hipMemcpyAsync(out, at<float>(x, x->lay.logits) + (size_t)first * x->cfg.vocab, 4ull * count * x->cfg.vocab,
                         hipMemcpyDeviceToHost, x->sA));
  HIP_TRY(hipStreamSynchronize(x->sA));
  return PPSD_OK;
}

int ppsd_read_drafts(ppsd_ctx *x, int32_t first, int32_t count, int32_t *out) {
  if (!x || !out) return fail(PPSD_EARG, "null argument");
  if (first < 0 || count < 0 || first + count > x->cfg.max_seq)
    return fail(PPSD_EARG, "rows %d..%d are outside the draft log", first, first + count - 1);
  HIP_TRY(hipMemcpyAsync(out, at<int32_t>(x, x->lay.drafts) + first, 4ull * count, hipMemcpyDeviceToHost, x->sA));
  HIP_TRY(hipStreamSynchronize(x->sA));
  return PPSD_OK;
}

int ppsd_launch_info(const ppsd_ctx *x, ppsd_launch_info_t *out) {
  if (!x || !out) return fail(PPSD_EARG, "null argument");
  const ppsd_config &c = x->cfg;
  out->compute_units = x->n_cu;
  out->attn_splits = x->lay.n_splits;
  out->prefill_matrix_core = x->lay.pf ? 1 : 0;
  out->prefill_chunk = x->lay.pf ? x->lay.pf_chunk : 0;
  out->grid_qkv = x->gemv_grid((c.n_heads + 2 * c.n_kv_heads) * (c.head_dim / 2));
  out->grid_proj = x->gemv_grid(c.d_model);
  out->grid_gate_up = x->gemv_grid(c.d_ffn, kGateUpWgsPerCu);
  out->grid_head = x->cm.dm.head_blocks;
  out->draft_share_of_256 = x->cm.dm.draft_share;
  out->streams = c.mode == PPSD_MODE_PIPELINE ? x->n_streams : c.mode == PPSD_MODE_OVERLAP ? 2 : 1;
  out->pipeline_stages = x->cm.dm.n_stages;
  out->eesd_gamma = x->gamma;
  return PPSD_OK;
}

int ppsd_kernel_times(const ppsd_ctx *x, ppsd_kernel_times_t *out) {
  if (!x || !out) return fail(PPSD_EARG, "null argument");
  if (!x->cfg.time_kernels) return fail(PPSD_ESTATE, "context was not created with time_kernels = 1");
  *out = x->ktimes;
  return PPSD_OK;
}

int ppsd_trace_request(ppsd_ctx *x, int32_t step, int32_t workgroup) {
  if (!x) return fail(PPSD_EARG, "null argument");
  if (x->cfg.engine != PPSD_ENGINE_PERSISTENT) return fail(PPSD_ESTATE, "the timeline exists for the persistent engine only");
  x->trace_step = step;
  x->trace_wg = workgroup;
  return PPSD_OK;
}

int ppsd_trace_read(ppsd_ctx *x, int32_t n_phases, uint64_t *out) {
  if (!x || !out) return fail(PPSD_EARG, "null argument");
  if (n_phases < 0 || n_phases > kTracePhases) return fail(PPSD_EARG, "at most %d phases are recorded", kTracePhases);
  HIP_TRY(hipMemcpyAsync(out, at<uint64_t>(x, x->lay.trace), 8ull * kTraceSlots * n_phases, hipMemcpyDeviceToHost, x->sA));
  HIP_TRY(hipStreamSynchronize(x->sA));
  return PPSD_OK;
}

int ppsd_hbm_read_probe(const void *buf, size_t bytes, void *stream, int32_t iters, float *avg_ms) {
  if (!buf || !avg_ms || iters < 1 || bytes < 16 || (uintptr_t)buf % 16) return fail(PPSD_EARG, "bad probe argument");
  hipStream_t s = (hipStream_t)stream;
  static uint32_t *s_sink = nullptr;   // the probe never writes in practice, but needs a valid target
  if (!s_sink) HIP_TRY(hipHostMalloc((void **)&s_sink, 64, hipHostMallocDefault));
  uint32_t *sink = s_sink;
  const size_t n_vec = bytes / 16;
  int dev = 0, n_cu = 0;
  HIP_TRY(hipGetDevice(&dev));
  HIP_TRY(hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev));
  const int blocks = n_cu;                  // one resident workgroup per compute unit
  struct Events {                           // destroyed on every return path
    hipEvent_t a = nullptr, b = nullptr;
    ~Events() { if (a) (void)hipEventDestroy(a); if (b) (void)hipEventDestroy(b); }
  } ev;
  HIP_TRY(hipEventCreate(&ev.a));
  HIP_TRY(hipEventCreate(&ev.b));
  hipEvent_t e0 = ev.a, e1 = ev.b;
  hipLaunchKernelGGL(k_read_probe, dim3(blocks), dim3(kGBlock), 0, s, (const uint4 *)buf, n_vec, sink);   // warm-up
  HIP_TRY(hipEventRecord(e0, s));
  for (int k = 0; k < iters; ++k) hipLaunchKernelGGL(k_read_probe, dim3(blocks), dim3(kGBlock), 0, s, (const uint4 *)buf, n_vec, sink);
  HIP_TRY(hipEventRecord(e1, s));
  HIP_TRY(hipStreamSynchronize(s));
  HIP_TRY(hipGetLastError());
  float ms = 0.f;
  HIP_TRY(hipEventElapsedTime(&ms, e0, e1));
  *avg_ms = ms / iters;
  return PPSD_OK;
}

}  // extern "C"
