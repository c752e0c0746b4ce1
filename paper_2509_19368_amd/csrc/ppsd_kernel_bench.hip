// Kernel-level benchmark of the weight-streaming kernels at a model shape, without Python or torch:
// each kernel is launched back to back over weight regions that rotate through a multi-GiB buffer
// (so no launch finds its weights in a cache), in the library's own launch configuration, with the
// device state set to "active".  Prints microseconds per launch and the algorithmic GB/s.
// Also the reference dispatches for scaling rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE readings:
// k_read_probe over 1 GiB and a 1 GiB device-to-device copy.
//
// usage: ppsd_kernel_bench [d_model d_ffn vocab n_heads n_kv_heads head_dim [iters [context [splits [passes]]]]]   (bf16 storage)
// With a context length > 0, the decode attention kernel is timed too: one query over `context` cached positions,
// 32 layers' worth of K/V pages visited in turn (so no launch finds its rows in a cache), head_dim 128 only.
// With passes > 0, the four batched projections are also launched in the order of the verify pass (24 layers per
// pass), so that a kernel trace of this program shows each kernel between its real neighbours.
#include <cstdio>
#include <cstdlib>

#include "ppsd_batch.h"

using namespace ppsd;

#define CK(x)                                                                                       \
  do {                                                                                              \
    hipError_t e_ = (x);                                                                            \
    if (e_ != hipSuccess) { printf("HIP error %s at %s:%d\n", hipGetErrorString(e_), __FILE__, __LINE__); return 1; } \
  } while (0)

__global__ void k_copy16(const uint4 *src, uint4 *dst, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) dst[i] = src[i];
}

// bf16 values spread over (-0.04, 0.04) from a hash of the index: weights whose bits vary like a model's
__global__ void k_fill_bf16(bf16_t *w, size_t n, unsigned seed) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) {
    unsigned long long z = (i + seed) * 0x9E3779B97F4A7C15ull;
    z ^= z >> 29; z *= 0xBF58476D1CE4E5B9ull; z ^= z >> 32;
    w[i] = float_to_bf16_rne(((int)(z & 0xffff) - 32768) * (0.04f / 32768.f));
  }
}
__global__ void k_fill_f32(float *p, size_t n, unsigned seed) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) {
    unsigned long long z = (i + seed) * 0x9E3779B97F4A7C15ull;
    z ^= z >> 29; z *= 0xBF58476D1CE4E5B9ull; z ^= z >> 32;
    p[i] = ((int)(z & 0xffff) - 32768) * (1.0f / 32768.f);
  }
}

int main(int argc, char **argv) {
  int d = 4096, f = 11008, V = 32000, n_h = 32, n_kv = 32, hd = 128, iters = 30;
  if (argc >= 7) { d = atoi(argv[1]); f = atoi(argv[2]); V = atoi(argv[3]); n_h = atoi(argv[4]); n_kv = atoi(argv[5]); hd = atoi(argv[6]); }
  if (argc >= 8) iters = atoi(argv[7]);
  const int ctx = argc >= 9 ? atoi(argv[8]) : 0;
  const int ctx_splits = argc >= 10 ? atoi(argv[9]) : 0;
  const int seq_reps = argc >= 11 ? atoi(argv[10]) : 0;
  const int nq = n_h * hd;
  if (d % 8 || f % 8 || d > 8192 || f > 16384 || nq > 16384 || (hd != 64 && hd != 128)) { printf("unsupported shape\n"); return 2; }
  int dev = 0, n_cu = 0;
  CK(hipGetDevice(&dev));
  CK(hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev));
  const size_t bytes = (size_t)6 << 30;
  char *W, *ws;
  CK(hipMalloc(&W, bytes));
  const bool varied = getenv("PPSD_BENCH_CONSTANT_DATA") == nullptr;
  if (varied) hipLaunchKernelGGL(k_fill_bf16, dim3(8192), dim3(256), 0, 0, (bf16_t *)W, bytes / 2, 11u);
  else CK(hipMemset(W, 0x3c, bytes));      // bf16 0x3c3c = 0.0115: finite products
  CK(hipMalloc(&ws, (size_t)64 << 20));
  CK(hipMemset(ws, 0, (size_t)64 << 20));
  if (varied) {                             // activations, gains and staged inputs: values in (-1, 1)
    hipLaunchKernelGGL(k_fill_f32, dim3(1024), dim3(256), 0, 0, (float *)(ws + (1 << 20)), (size_t)(1 << 20) / 4, 3u);
    hipLaunchKernelGGL(k_fill_f32, dim3(1024), dim3(256), 0, 0, (float *)(ws + (5 << 20)), (size_t)(3 << 20) / 4, 5u);
    hipLaunchKernelGGL(k_fill_f32, dim3(1024), dim3(256), 0, 0, (float *)(ws + (44 << 20)), (size_t)(4 << 20) / 4, 7u);
  }
  CK(hipDeviceSynchronize());
  Common c{};
  c.st = (DevState *)ws;
  c.prompt = (int32_t *)(ws + 4096);
  c.xbuf = (float *)(ws + (1 << 20));
  c.rope_cos = (float *)(ws + (2 << 20));
  c.rope_sin = (float *)(ws + (3 << 20));
  c.page_table = (int32_t *)(ws + (4 << 20));
  c.kv_pool = ws + (8 << 20);
  const int max_seq = 386, pt = 16, n_pages = (max_seq + pt - 1) / pt;
  c.dm = Dims{d, n_h, n_kv, hd, f, V, 32, 8, max_seq, pt, n_pages, 1, 0, gemv_grid_for((V + 1) / 2, n_cu, kGemvWgsPerCu), 4, 4 /* log2(pt) */, 1e-5f, 0.088f};
  DevState st{};
  st.t = 10; st.last_token = 5; st.full = 1; st.draft = 7; st.n_out = 0; st.target = 1 << 30;
  CK(hipMemcpy(ws, &st, sizeof st, hipMemcpyHostToDevice));
  float *gain = (float *)(ws + (5 << 20)), *mout = (float *)(ws + (6 << 20)), *vin = (float *)(ws + (7 << 20));
  float2 *cand = (float2 *)(ws + (40 << 20));
  hipEvent_t e0, e1;
  CK(hipEventCreate(&e0));
  CK(hipEventCreate(&e1));
  printf("device: %d CUs; shape d=%d f=%d V=%d heads=%d/%d x %d; %d launches each\n", n_cu, d, f, V, n_h, n_kv, hd, iters);

  // reference dispatches for counter scaling
  {
    const size_t gib = (size_t)1 << 30;
    hipLaunchKernelGGL(k_read_probe, dim3(n_cu), dim3(kGBlock), 0, 0, (const uint4 *)W, gib / 16, (uint32_t *)(ws + (50 << 20)));
    hipLaunchKernelGGL(k_copy16, dim3(4096), dim3(256), 0, 0, (const uint4 *)W, (uint4 *)(W + 2 * gib), gib / 16);
    CK(hipDeviceSynchronize());
    printf("reference dispatches: k_read_probe reads 1 GiB; k_copy16 reads 1 GiB and writes 1 GiB\n");
  }

  auto run = [&](const char *name, size_t mat_bytes, auto launch) {
    const int parts = (int)(bytes / mat_bytes);
    for (int i = 0; i < 3; ++i) launch((const bf16_t *)(W + (size_t)(i % parts) * mat_bytes));
    (void)hipDeviceSynchronize();
    (void)hipEventRecord(e0);
    for (int i = 0; i < iters; ++i) launch((const bf16_t *)(W + (size_t)((i + 3) % parts) * mat_bytes));
    (void)hipEventRecord(e1);
    (void)hipEventSynchronize(e1);
    float ms = 0.f;
    (void)hipEventElapsedTime(&ms, e0, e1);
    ms /= iters;
    printf("%-22s %7.1f MB  %7.2f us/launch  %6.0f GB/s\n", name, mat_bytes / 1e6, ms * 1e3, mat_bytes / ms / 1e6);
    fflush(stdout);
  };
  const int qkv_rows = (n_h + 2 * n_kv) * hd;
  run("k_qkv", (size_t)qkv_rows * d * 2, [&](const bf16_t *w) {
    hipLaunchKernelGGL((k_qkv<bf16_t>), dim3(gemv_grid_for(qkv_rows / 2, n_cu, kGemvWgsPerCu)), dim3(kGBlock), (size_t)xs_floats(2, d) * 4, 0, c,
                       (int)kVanilla, 3, (int)kXDraft, 0, w, gain, w, mout);
  });
  run("k_proj_resid (o_proj)", (size_t)d * nq * 2, [&](const bf16_t *w) {
    hipLaunchKernelGGL((k_proj_resid<bf16_t>), dim3(gemv_grid_for(d, n_cu, kGemvWgsPerCu)), dim3(kGBlock), (size_t)xs_floats(2, nq) * 4, 0, c,
                       (int)kVanilla, vin, nq, w, d, (int)kXDraft, (int)kXDraft);
  });
  run("k_gate_up", (size_t)2 * f * d * 2, [&](const bf16_t *w) {
    hipLaunchKernelGGL((k_gate_up<bf16_t>), dim3(gemv_grid_for(f, n_cu, kGateUpWgsPerCu)), dim3(kGBlock), (size_t)xs_floats(2, d) * 4, 0, c,
                       (int)kVanilla, (int)kXDraft, gain, w, mout);
  });
  run("k_proj_resid (down)", (size_t)d * f * 2, [&](const bf16_t *w) {
    hipLaunchKernelGGL((k_proj_resid<bf16_t>), dim3(gemv_grid_for(d, n_cu, kGemvWgsPerCu)), dim3(kGBlock), (size_t)xs_floats(2, f) * 4, 0, c,
                       (int)kVanilla, vin, f, w, d, (int)kXDraft, (int)kXDraft);
  });
  run("k_head", (size_t)V * d * 2, [&](const bf16_t *w) {
    hipLaunchKernelGGL((k_head<bf16_t>), dim3(c.dm.head_blocks), dim3(kGBlock), (size_t)xs_floats(2, d) * 4, 0, c, (int)kVanilla, (int)kXDraft, gain,
                       w, cand, (float *)nullptr, 1, (float *)nullptr);
  });

  // decode attention at a long context
  if (ctx > 0 && hd == 128 && (n_h / n_kv == 1 || n_h / n_kv == 2 || n_h / n_kv == 4) && n_h % n_kv == 0) {
    const int a_layers = 32, a_pages = (ctx + pt - 1) / pt;
    int a_splits = ctx_splits > 0 ? ctx_splits : (ctx <= 512 ? 1 : (ctx + 511) / 512);
    if (a_splits > kMaxAttnSplits) a_splits = kMaxAttnSplits;
    if (a_pages > kAttnLdsPages) { printf("context too long for this benchmark\n"); return 2; }
    const size_t layer_bytes = (size_t)a_pages * n_kv * 2 * pt * hd * 2;
    char *kvp; int32_t *ptab; float *apart; int *acount;
    CK(hipMalloc(&kvp, layer_bytes * a_layers));
    CK(hipMemset(kvp, 0x3c, layer_bytes * a_layers));
    CK(hipMalloc(&ptab, 4 * (size_t)a_pages));
    CK(hipMalloc(&apart, 4 * (size_t)n_h * kMaxAttnSplits * (hd + 2)));
    CK(hipMalloc(&acount, 4 * (size_t)kCounterStride * n_kv));
    CK(hipMemset(acount, 0, 4 * (size_t)kCounterStride * n_kv));
    {
      int32_t *h = (int32_t *)malloc(4 * (size_t)a_pages);
      for (int i = 0; i < a_pages; ++i) h[i] = i;
      CK(hipMemcpy(ptab, h, 4 * (size_t)a_pages, hipMemcpyHostToDevice));
      free(h);
    }
    Common ca = c;
    ca.page_table = ptab; ca.kv_pool = kvp;
    ca.dm.max_seq = a_pages * pt; ca.dm.n_pages = a_pages; ca.dm.n_splits = a_splits; ca.dm.L = a_layers;
    DevState sa = st;
    sa.t = ctx - 1;
    CK(hipMemcpy(ws, &sa, sizeof sa, hipMemcpyHostToDevice));
    const size_t kv_read = (size_t)ctx * n_kv * 2 * hd * 2;
    int turn = 0;
    char name[64];
    snprintf(name, sizeof name, "k_attn ctx %d x%d", ctx, a_splits);
    run(name, kv_read, [&](const bf16_t *) {
      const int layer = turn++ % a_layers;
      const dim3 grid(n_kv, a_splits);
      const int G = n_h / n_kv;
      if (G == 1) hipLaunchKernelGGL((k_attn<bf16_t, 128, 1>), grid, dim3(kGBlock), 0, 0, ca, (int)kVanilla, layer, (const float *)vin, mout, apart, acount);
      else if (G == 2) hipLaunchKernelGGL((k_attn<bf16_t, 128, 2>), grid, dim3(kGBlock), 0, 0, ca, (int)kVanilla, layer, (const float *)vin, mout, apart, acount);
      else hipLaunchKernelGGL((k_attn<bf16_t, 128, 4>), grid, dim3(kGBlock), 0, 0, ca, (int)kVanilla, layer, (const float *)vin, mout, apart, acount);
    });
    CK(hipMemcpy(ws, &st, sizeof st, hipMemcpyHostToDevice));
    CK(hipGetLastError());
  }

  // the batched verify pass of draft-then-verify rounds, four tokens (same matrices, streamed once)
  constexpr int B = 4;
  const int lds_cap = 150 * 1024;
  CK(hipFuncSetAttribute((const void *)k_qkv_b<bf16_t, B>, hipFuncAttributeMaxDynamicSharedMemorySize, lds_cap));
  CK(hipFuncSetAttribute((const void *)k_gate_up_b<bf16_t, B>, hipFuncAttributeMaxDynamicSharedMemorySize, lds_cap));
  CK(hipFuncSetAttribute((const void *)k_head_b<bf16_t, B>, hipFuncAttributeMaxDynamicSharedMemorySize, lds_cap));
  CK(hipFuncSetAttribute((const void *)k_proj_resid_b<bf16_t, B>, hipFuncAttributeMaxDynamicSharedMemorySize, lds_cap));
  if ((size_t)B * xs_floats(2, d) * 4 > (size_t)lds_cap) { printf("batched kernels skipped: %d x d_model floats exceed the LDS\n", B); return 0; }
  auto bgrid = [&](int n_tasks, size_t lds, int per_cu) {
    int fit = (int)((160 * 1024) / (lds + 1024));
    if (fit < 1) fit = 1;
    return gemv_grid_for(n_tasks, n_cu, fit < per_cu ? fit : per_cu);
  };
  float *vb = (float *)(ws + (44 << 20)), *mb = (float *)(ws + (46 << 20));
  float2 *candb = (float2 *)(ws + (48 << 20));
  const size_t lds_d = (size_t)B * xs_floats(2, d) * 4;
  run("k_qkv_b<4>", (size_t)qkv_rows * d * 2, [&](const bf16_t *w) {
    hipLaunchKernelGGL((k_qkv_b<bf16_t, B>), dim3(bgrid(qkv_rows / 2, lds_d, kGemvWgsPerCu)), dim3(kGBlock), lds_d, 0, c, 3,
                       (int)kXBatchInSlot0, gain, w, vb);
  });
  run("k_gate_up_b<4>", (size_t)2 * f * d * 2, [&](const bf16_t *w) {
    hipLaunchKernelGGL((k_gate_up_b<bf16_t, B>), dim3(bgrid(f, lds_d, kGateUpWgsPerCu)), dim3(kGBlock), lds_d, 0, c,
                       (int)kXBatchWorkSlot0, gain, w, mb);
  });
  CK(hipFuncSetAttribute((const void *)k_proj_resid_bs<bf16_t, B>, hipFuncAttributeMaxDynamicSharedMemorySize, lds_cap));
  run("k_proj_resid_bs<4> (down)", (size_t)d * f * 2, [&](const bf16_t *w) {
    // as the library launches it: column slabs of at most 64 KB of staged inputs, walked inside one launch
    const int n_slabs = (int)(((size_t)B * f * 4 + 65535) / 65536);
    const int Cs = ((f + n_slabs - 1) / n_slabs + 511) / 512 * 512;
    if (Cs < f) {
      hipLaunchKernelGGL((k_proj_resid_bs<bf16_t, B>), dim3((d + kGWaves - 1) / kGWaves), dim3(kGBlock), (size_t)B * xs_floats(2, Cs) * 4, 0, c,
                         (const float *)mb, f, Cs, w, d, (int)kXBatchWorkSlot0, (int)kXBatchWorkSlot0);
    } else {
      const size_t lds = (size_t)B * xs_floats(2, f) * 4;
      hipLaunchKernelGGL((k_proj_resid_b<bf16_t, B>), dim3(bgrid((d + 1) / 2, lds, kGemvWgsPerCu)), dim3(kGBlock), lds, 0, c,
                         (const float *)mb, f, 0, f, w, d, (int)kXBatchWorkSlot0, (int)kXBatchWorkSlot0);
    }
  });
  run("k_head_b<4>", (size_t)V * d * 2, [&](const bf16_t *w) {
    hipLaunchKernelGGL((k_head_b<bf16_t, B>), dim3(c.dm.head_blocks), dim3(kGBlock), lds_d, 0, c, (int)kXBatchWorkSlot0, gain, w,
                       candb, (float *)nullptr, (float *)nullptr);
  });
  CK(hipGetLastError());

  // the batched kernels in the order of the verify pass (QKV, o_proj, gate/up, down per layer), every launch
  // on fresh weights: what a kernel costs between its real neighbours, for a kernel trace of this program
  if (seq_reps > 0) {
    const size_t per_layer = ((size_t)qkv_rows * d + (size_t)d * nq + (size_t)2 * f * d + (size_t)d * f) * 2;
    const int seq_layers = 24, parts = (int)(bytes / per_layer);
    const size_t lds_o = (size_t)B * xs_floats(2, nq) * 4;
    const int n_slabs = (int)(((size_t)B * f * 4 + 65535) / 65536);
    const int Cs = ((f + n_slabs - 1) / n_slabs + 511) / 512 * 512;
    if (Cs >= f || lds_o > 65536) { printf("sequence skipped: it covers shapes whose down-projection is walked in slabs\n"); return 0; }
    int turn = 0;
    auto layer = [&]() {
      const bf16_t *w = (const bf16_t *)(W + (size_t)(turn++ % parts) * per_layer);
      hipLaunchKernelGGL((k_qkv_b<bf16_t, B>), dim3(bgrid(qkv_rows / 2, lds_d, kGemvWgsPerCu)), dim3(kGBlock), lds_d, 0, c, 3,
                         (int)kXBatchInSlot0, gain, w, vb);
      w += (size_t)qkv_rows * d;
      hipLaunchKernelGGL((k_proj_resid_b<bf16_t, B>), dim3(bgrid((d + 1) / 2, lds_o, kGemvWgsPerCu)), dim3(kGBlock), lds_o, 0, c,
                         (const float *)vb, nq, 0, nq, w, d, (int)kXBatchWorkSlot0, (int)kXBatchWorkSlot0);
      w += (size_t)d * nq;
      hipLaunchKernelGGL((k_gate_up_b<bf16_t, B>), dim3(bgrid(f, lds_d, kGateUpWgsPerCu)), dim3(kGBlock), lds_d, 0, c,
                         (int)kXBatchWorkSlot0, gain, w, mb);
      w += (size_t)2 * f * d;
      hipLaunchKernelGGL((k_proj_resid_bs<bf16_t, B>), dim3((d + kGWaves - 1) / kGWaves), dim3(kGBlock), (size_t)B * xs_floats(2, Cs) * 4, 0, c,
                         (const float *)mb, f, Cs, w, d, (int)kXBatchWorkSlot0, (int)kXBatchWorkSlot0);
    };
    for (int l = 0; l < seq_layers; ++l) layer();
    CK(hipDeviceSynchronize());
    CK(hipEventRecord(e0));
    for (int r = 0; r < seq_reps; ++r)
      for (int l = 0; l < seq_layers; ++l) layer();
    CK(hipEventRecord(e1));
    CK(hipEventSynchronize(e1));
    float ms = 0.f;
    CK(hipEventElapsedTime(&ms, e0, e1));
    printf("verify-pass sequence (4 launches per layer, %d layers, %d passes): %.2f us per layer\n", seq_layers, seq_reps,
           ms * 1e3 / seq_reps / seq_layers);
    CK(hipGetLastError());
  }
  return 0;
}
