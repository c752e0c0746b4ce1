// ppsd_cli: a plain C++ program (no Python, no torch) that drives libppsd.so through include/ppsd.h only.
//
// It allocates device memory itself, fills a model of one of the workload shapes from a counter-based hash
// (zero-mean bell-shaped values of standard deviation 0.02, gains 1, exit head = a separately stored copy of
// the LM head, W_o / W_down of the layers behind the exit layer scaled by `damp`), runs ppsd_prefill and
// ppsd_decode and prints tokens/s, the counters of ppsd_stats and the launch configuration.  It is the program
// to put behind `rocprofv3 --kernel-trace --stats --` and `rocprofv3 --pmc FETCH_SIZE --` so that timings and
// HBM counters come from the library's own kernels, and it exercises the C ABI from the C side (`--check`
// decodes in every schedule and requires one token stream: the method is lossless, Sec. 5.1).
//
//   ppsd_cli <C1|C2|C4|C5|7B_E4|7B_E16> [--mode vanilla|serial|overlap|pipeline|eesd] [--prompt N] [--decode N]
//            [--gens K] [--damp X] [--exit-layer E] [--later-stage W] [--capacity-for-decode N] [--check] [--calibrate]
//            [--static-scratch] [--no-graph]
//   --later-stage W: PPSD_MODE_PIPELINE with the layers behind the draft stage in stages of W layers.
//   --capacity-for-decode N: size max_seq as if N tokens were decoded (a short counter run then keeps the
//   attention split count of the full workload).
#include <hip/hip_runtime.h>

#include <chrono>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <string>
#include <vector>

#include "../../include/ppsd.h"

#define CK(expr)                                                                                   \
  do {                                                                                             \
    hipError_t e_ = (expr);                                                                        \
    if (e_ != hipSuccess) { fprintf(stderr, "%s: %s\n", #expr, hipGetErrorString(e_)); exit(3); }  \
  } while (0)
#define PK(expr)                                                                                   \
  do {                                                                                             \
    int rc_ = (expr);                                                                              \
    if (rc_ != PPSD_OK) { fprintf(stderr, "%s -> %d: %s\n", #expr, rc_, ppsd_last_error()); exit(4); } \
  } while (0)

namespace {

struct Shape {
  const char *name;
  int L, E, d, n_h, n_kv, hd, f, V, dtype;
  float rope_base, damp;
  int prompt, decode;
};

// The workload list's shapes: tiny fp32; Llama-2-7B; Llama-2-13B; Llama-3-8B (GQA, long context); the 7B
// shape at the other two exit layers of the granularity grid.
const Shape kShapes[] = {
    {"C1", 4, 1, 256, 4, 4, 64, 688, 2048, PPSD_FP32, 1.0e4f, 0.1f, 16, 64},
    {"C2", 32, 8, 4096, 32, 32, 128, 11008, 32000, PPSD_BF16, 1.0e4f, 0.04f, 128, 256},
    {"C4", 40, 10, 5120, 40, 40, 128, 13824, 32000, PPSD_BF16, 1.0e4f, 0.0548f, 512, 512},
    {"C5", 32, 8, 4096, 32, 8, 128, 14336, 128256, PPSD_BF16, 5.0e5f, 0.0548f, 8192, 512},
    {"7B_E4", 32, 4, 4096, 32, 32, 128, 11008, 32000, PPSD_BF16, 1.0e4f, 0.0548f, 256, 256},
    {"7B_E16", 32, 16, 4096, 32, 32, 128, 11008, 32000, PPSD_BF16, 1.0e4f, 0.1481f, 256, 256},
};

__device__ __host__ inline unsigned long long mix64(unsigned long long z) {
  z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ull;
  z ^= z >> 27; z *= 0x94D049BB133111EBull;
  z ^= z >> 31;
  return z;
}

// Element i of tensor `tag`: scale * (centred sum of four 16-bit fields of a hash) / its standard deviation.
__device__ inline float bell(unsigned long long tag, size_t i, float scale) {
  const unsigned long long z = mix64(tag * 0xD6E8FEB86659FD93ull + (unsigned long long)i * 0x9E3779B97F4A7C15ull);
  const int s = (int)(z & 0xffff) + (int)((z >> 16) & 0xffff) + (int)((z >> 32) & 0xffff) + (int)(z >> 48) - 2 * 65535;
  return (float)s * (scale / 37837.2f);     // sqrt(4 * (65536^2 - 1) / 12)
}

__device__ inline unsigned short to_bf16(float f) {
  unsigned u = __float_as_uint(f);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (unsigned short)(u >> 16);
}

__global__ void k_fill_bf16(unsigned short *p, size_t n, unsigned long long tag, float scale) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = to_bf16(bell(tag, i, scale));
}
__global__ void k_fill_f32(float *p, size_t n, unsigned long long tag, float scale) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = bell(tag, i, scale);
}
__global__ void k_fill_const(float *p, size_t n, float v) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = v;
}
// Reference dispatch of known size for scaling counter readings: reads n and writes n 16-byte vectors.
__global__ void k_copy16(const uint4 *src, uint4 *dst, size_t n) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) dst[i] = src[i];
}

std::vector<void *> g_allocs;
void *dmalloc(size_t bytes) {
  void *p = nullptr;
  CK(hipMalloc(&p, bytes));
  g_allocs.push_back(p);
  return p;
}

void *matrix(const Shape &s, unsigned long long tag, size_t rows, size_t cols, float scale) {
  const size_t n = rows * cols;
  void *p = dmalloc(n * (s.dtype == PPSD_FP32 ? 4 : 2));
  if (s.dtype == PPSD_FP32) hipLaunchKernelGGL(k_fill_f32, dim3(2048), dim3(256), 0, 0, (float *)p, n, tag, scale);
  else hipLaunchKernelGGL(k_fill_bf16, dim3(2048), dim3(256), 0, 0, (unsigned short *)p, n, tag, scale);
  return p;
}
void *gains(int d) {
  float *p = (float *)dmalloc(4ull * d);
  hipLaunchKernelGGL(k_fill_const, dim3(8), dim3(256), 0, 0, p, (size_t)d, 1.0f);
  return p;
}

struct Model {
  Shape s;
  void *embed, *final_norm, *lm_head, *exit_norm, *exit_head;
  std::vector<const void *> attn_norm, wqkv, wo, mlp_norm, wgu, wdown;
};

Model make_model(const Shape &s) {
  Model m;
  m.s = s;
  const size_t d = s.d, nq = (size_t)s.n_h * s.hd, qkv_rows = (size_t)(s.n_h + 2 * s.n_kv) * s.hd;
  m.embed = matrix(s, 1, s.V, d, 0.02f);
  m.lm_head = matrix(s, 2, s.V, d, 0.02f);
  m.exit_head = dmalloc((size_t)s.V * d * (s.dtype == PPSD_FP32 ? 4 : 2));
  CK(hipMemcpy(m.exit_head, m.lm_head, (size_t)s.V * d * (s.dtype == PPSD_FP32 ? 4 : 2), hipMemcpyDeviceToDevice));
  m.final_norm = gains(s.d);
  m.exit_norm = gains(s.d);
  for (int l = 0; l < s.L; ++l) {
    const float out_scale = 0.02f * (l >= s.E ? s.damp : 1.0f);
    const unsigned long long t = 16ull * (l + 1);
    m.attn_norm.push_back(gains(s.d));
    m.wqkv.push_back(matrix(s, t + 0, qkv_rows, d, 0.02f));
    m.wo.push_back(matrix(s, t + 1, d, nq, out_scale));
    m.mlp_norm.push_back(gains(s.d));
    m.wgu.push_back(matrix(s, t + 2, 2ull * s.f, d, 0.02f));
    m.wdown.push_back(matrix(s, t + 3, d, s.f, out_scale));
  }
  CK(hipDeviceSynchronize());
  return m;
}

struct RunResult {
  std::vector<int32_t> tokens;     // token #0 and the decoded ones (last generation)
  double tok_s = 0, prefill_ms = 0;
  ppsd_stats_t st{};
  ppsd_launch_info_t info{};
};

int mode_of(const std::string &m) {
  if (m == "vanilla") return PPSD_MODE_VANILLA;
  if (m == "serial") return PPSD_MODE_SERIAL;
  if (m == "overlap") return PPSD_MODE_OVERLAP;
  if (m == "pipeline") return PPSD_MODE_PIPELINE;
  if (m == "eesd") return PPSD_MODE_EESD;
  fprintf(stderr, "unknown mode %s\n", m.c_str());
  exit(2);
}

int g_later_stage = 0, g_capacity_decode = 0;

RunResult run(const Model &m, int mode, int n_prompt, int n_decode, int gens, bool graph, bool static_scratch,
              hipStream_t sA, hipStream_t sB) {
  const Shape &s = m.s;
  ppsd_config c;
  memset(&c, 0, sizeof c);
  c.n_layers = s.L; c.exit_layer = s.E; c.d_model = s.d; c.n_heads = s.n_h; c.n_kv_heads = s.n_kv; c.head_dim = s.hd;
  c.d_ffn = s.f; c.vocab = s.V; c.dtype = s.dtype; c.kv_page_tokens = 16; c.mode = mode;
  const int stages = (s.L + s.E - 1) / s.E;
  c.max_seq = n_prompt + 1 + (g_capacity_decode > n_decode ? g_capacity_decode : n_decode) + (stages - 1 > 4 ? stages - 1 : 4);
  c.pipeline_stage_layers = g_later_stage;
  c.rope_base = s.rope_base; c.rms_eps = 1e-5f; c.use_graph = graph ? 1 : 0;
  const size_t ws_bytes = ppsd_workspace_bytes(&c);
  if (!ws_bytes) { fprintf(stderr, "ppsd_workspace_bytes: %s\n", ppsd_last_error()); exit(4); }
  void *ws = nullptr;
  CK(hipMalloc(&ws, ws_bytes));
  ppsd_buffers b;
  memset(&b, 0, sizeof b);
  b.embed = m.embed; b.final_norm = m.final_norm; b.lm_head = m.lm_head; b.exit_norm = m.exit_norm; b.exit_head = m.exit_head;
  b.attn_norm = m.attn_norm.data(); b.wqkv = m.wqkv.data(); b.wo = m.wo.data(); b.mlp_norm = m.mlp_norm.data();
  b.wgu = m.wgu.data(); b.wdown = m.wdown.data();
  b.workspace = ws; b.workspace_bytes = ws_bytes; b.stream_draft = sA; b.stream_verify = sB;
  ppsd_ctx *ctx = nullptr;
  PK(ppsd_load_weights(&c, &b, &ctx));
  std::vector<int32_t> prompt(n_prompt);
  for (int i = 0; i < n_prompt; ++i) prompt[i] = (int32_t)(mix64(0x5151ull + (unsigned long long)i * 0x9E3779B97F4A7C15ull) % (unsigned long long)s.V);
  RunResult r;
  r.tokens.assign(n_decode + 1, -1);
  double best = 1e30;
  for (int g = 0; g < gens; ++g) {
    auto t0 = std::chrono::steady_clock::now();
    PK(ppsd_prefill(ctx, prompt.data(), n_prompt, &r.tokens[0]));
    auto t1 = std::chrono::steady_clock::now();
    int32_t nw = 0;
    if (static_scratch) PK(ppsd_decode_static_scratch(ctx, n_decode, r.tokens.data() + 1, &nw));
    else PK(ppsd_decode(ctx, n_decode, r.tokens.data() + 1, &nw));
    auto t2 = std::chrono::steady_clock::now();
    if (nw != n_decode) { fprintf(stderr, "ppsd_decode wrote %d of %d tokens\n", nw, n_decode); exit(5); }
    const double dt = std::chrono::duration<double>(t2 - t1).count();
    if (g > 0 || gens == 1) best = dt < best ? dt : best;
    r.prefill_ms = 1e3 * std::chrono::duration<double>(t1 - t0).count();
  }
  r.tok_s = n_decode / best;
  PK(ppsd_stats(ctx, &r.st));
  PK(ppsd_launch_info(ctx, &r.info));
  ppsd_free(ctx);
  CK(hipFree(ws));
  return r;
}

}  // namespace

int main(int argc, char **argv) {
  if (argc < 2) {
    fprintf(stderr, "usage: %s <C1|C2|C4|C5|7B_E4|7B_E16> [--mode M] [--prompt N] [--decode N] [--gens K] [--damp X] "
                    "[--exit-layer E] [--later-stage W] [--capacity-for-decode N] [--check] [--calibrate] [--static-scratch] "
                    "[--no-graph]\n", argv[0]);
    return 2;
  }
  const Shape *found = nullptr;
  for (const Shape &s : kShapes) if (!strcmp(s.name, argv[1])) found = &s;
  if (!found) { fprintf(stderr, "unknown workload %s\n", argv[1]); return 2; }
  Shape s = *found;
  setvbuf(stdout, nullptr, _IOLBF, 0);      // progress lines appear as they are printed, also in a redirected log
  std::string mode = "overlap";
  int gens = 2;
  bool check = false, calibrate = false, static_scratch = false, graph = true;
  for (int i = 2; i < argc; ++i) {
    const std::string a = argv[i];
    auto val = [&]() -> const char * { if (i + 1 >= argc) { fprintf(stderr, "%s needs a value\n", a.c_str()); exit(2); } return argv[++i]; };
    if (a == "--mode") mode = val();
    else if (a == "--prompt") s.prompt = atoi(val());
    else if (a == "--decode") s.decode = atoi(val());
    else if (a == "--gens") gens = atoi(val());
    else if (a == "--damp") s.damp = (float)atof(val());
    else if (a == "--exit-layer") s.E = atoi(val());
    else if (a == "--later-stage") g_later_stage = atoi(val());
    else if (a == "--capacity-for-decode") g_capacity_decode = atoi(val());
    else if (a == "--check") check = true;
    else if (a == "--calibrate") calibrate = true;
    else if (a == "--static-scratch") static_scratch = true;
    else if (a == "--no-graph") graph = false;
    else { fprintf(stderr, "unknown option %s\n", a.c_str()); return 2; }
  }
  if (s.prompt < 1 || s.decode < 1 || gens < 1) { fprintf(stderr, "prompt, decode and gens must be positive\n"); return 2; }
  hipStream_t sA, sB;
  CK(hipStreamCreateWithFlags(&sA, hipStreamNonBlocking));
  CK(hipStreamCreateWithFlags(&sB, hipStreamNonBlocking));
  if (calibrate) {
    const size_t n = (1ull << 30) / 16;
    uint4 *src = nullptr, *dst = nullptr;
    CK(hipMalloc((void **)&src, n * 16));
    CK(hipMalloc((void **)&dst, n * 16));
    CK(hipMemset(src, 0x5a, n * 16));
    for (int k = 0; k < 3; ++k) hipLaunchKernelGGL(k_copy16, dim3(4096), dim3(256), 0, 0, (const uint4 *)src, dst, n);
    CK(hipDeviceSynchronize());
    CK(hipFree(src));
    CK(hipFree(dst));
    printf("calibration: k_copy16 read 1 GiB and wrote 1 GiB, three dispatches\n");
  }
  printf("filling the model\n");
  const Model m = make_model(s);
  double bytes = 0;
  {
    const double es = s.dtype == PPSD_FP32 ? 4 : 2;
    const double layer = ((double)(s.n_h + 2 * s.n_kv) * s.hd * s.d + (double)s.d * s.n_h * s.hd + 3.0 * s.f * s.d) * es;
    bytes = s.L * layer + (double)s.V * s.d * es + 2.0 * s.L * s.n_kv * s.hd * es * (s.prompt + 1 + s.decode / 2.0);
  }
  printf("workload %s: %d layers, exit %d, d %d, heads %d/%d x %d, ffn %d, vocab %d, %s, prompt %d, decode %d, damp %g\n", s.name,
         s.L, s.E, s.d, s.n_h, s.n_kv, s.hd, s.f, s.V, s.dtype == PPSD_FP32 ? "fp32" : "bf16", s.prompt, s.decode, s.damp);
  int rc = 0;
  auto report = [&](const char *name, const RunResult &r) {
    const double alpha = r.st.drafts_compared ? (double)r.st.accepted / r.st.drafts_compared : 0.0;
    printf("%-8s %8.1f tok/s  %.3f of 8 TB/s per committed token  prefill %.1f ms  acceptance %.3f  (accepted %lld rejected %lld "
           "draft-only steps %lld ticks %lld rounds %lld)  [splits %d, prefill %s chunk %d, grids %d/%d/%d/%d, draft share %d/256, "
           "streams %d]\n", name, r.tok_s, r.tok_s * bytes / 8e12, r.prefill_ms, alpha, (long long)r.st.accepted,
           (long long)r.st.rejected, (long long)r.st.steps_draft_only, (long long)r.st.pipeline_ticks, (long long)r.st.eesd_rounds,
           r.info.attn_splits, r.info.prefill_matrix_core ? "mfma" : "looped", r.info.prefill_chunk, r.info.grid_qkv, r.info.grid_proj,
           r.info.grid_gate_up, r.info.grid_head, r.info.draft_share_of_256, r.info.streams);
    fflush(stdout);
  };
  if (check) {
    const char *names[] = {"vanilla", "serial", "overlap", "pipeline"};
    RunResult ref;
    for (int k = 0; k < 4; ++k) {
      if (k == 3 && (s.L + s.E - 1) / s.E > 16) continue;
      RunResult r = run(m, mode_of(names[k]), s.prompt, s.decode, gens, graph, static_scratch, sA, sB);
      report(names[k], r);
      if (k == 0) ref = r;
      else if (r.tokens != ref.tokens) { printf("MISMATCH: %s commits a different stream than vanilla\n", names[k]); rc = 1; }
    }
    printf(rc ? "check FAILED\n" : "check ok: every schedule commits vanilla decoding's stream\n");
  } else {
    RunResult r = run(m, mode_of(mode), s.prompt, s.decode, gens, graph, static_scratch, sA, sB);
    report(mode.c_str(), r);
  }
  for (void *p : g_allocs) CK(hipFree(p));
  CK(hipStreamDestroy(sA));
  CK(hipStreamDestroy(sB));
  return rc;
}
