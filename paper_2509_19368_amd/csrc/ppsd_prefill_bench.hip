// Kernel-level benchmark of the matrix-core prefill kernels at a model shape, without Python or torch:
// the four projections of a layer as the library launches them for one chunk of positions (GEMM, plus
// the reduce kernel when K is split) over weight regions that rotate through a multi-GiB buffer, and the
// attention kernel over the K/V rows the QKV projection wrote.  Prints microseconds per launch, the
// algorithmic TFLOP/s (2 M N K; attention: 2 M^2 hd n_heads, the causal half of QK^T and PV) and the
// rate the matrix cores run at (twice that: activations, queries and probabilities enter as bf16 high
// + low parts).
//
// usage: ppsd_prefill_bench [positions d_model d_ffn n_heads n_kv_heads [iters [tile]]]   (bf16 storage, head_dim 128;
//        tile = 1 or 2 forces the small or the big GEMM tile)
#include <algorithm>
#include <cstdio>
#include <cstdlib>

#include "ppsd_prefill.h"

using namespace ppsd;

#define CK(x)                                                                                       \
  do {                                                                                              \
    hipError_t e_ = (x);                                                                            \
    if (e_ != hipSuccess) { printf("HIP error %s at %s:%d\n", hipGetErrorString(e_), __FILE__, __LINE__); return 1; } \
  } while (0)

__global__ void k_fill_f32(float *p, size_t n, float v) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = v;
}

static int g_force_big = -1;

template <int EPI>
static void launch_gemm(const Common &c, PfGemm g, int n_cols) {
  pf_launch<EPI>(0, c, g, pf_plan(g.n_valid, n_cols, g.K, g_force_big));
}

int main(int argc, char **argv) {
  int M = 2048, d = 4096, f = 11008, n_h = 32, n_kv = 32, iters = 20;
  const int hd = 128;
  if (argc >= 6) { M = atoi(argv[1]); d = atoi(argv[2]); f = atoi(argv[3]); n_h = atoi(argv[4]); n_kv = atoi(argv[5]); }
  if (argc >= 7) iters = atoi(argv[6]);
  if (argc >= 8) g_force_big = atoi(argv[7]) == 2 ? 2 : 1;
  const int nq = n_h * hd, G = n_kv ? n_h / n_kv : 0, qkv_cols = (n_h + 2 * n_kv) * hd;
  if (M < 1 || M > kPfChunkMax || d % kPfBN || f % 64 || d % kPfBK || f % kPfBK || n_kv < 1 || n_h % n_kv || (G != 1 && G != 2 && G != 4) ||
      iters < 1) {
    printf("unsupported shape\n");
    return 2;
  }
  int dev = 0, n_cu = 0;
  CK(hipGetDevice(&dev));
  CK(hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev));
  const size_t wbytes = (size_t)4 << 30;
  const int pt = 16, n_pages = (M + pt - 1) / pt, mpad = (M + kPfBM - 1) / kPfBM * kPfBM;
  const size_t wide = (size_t)(d > nq ? d : nq), kmax = wide > (size_t)f ? wide : (size_t)f;
  size_t part = 0;
  part = std::max(part, pf_partial_floats(pf_plan(M, qkv_cols, d, g_force_big)));
  part = std::max(part, pf_partial_floats(pf_plan(M, d, nq, g_force_big)));
  part = std::max(part, pf_partial_floats(pf_plan(M, 2 * f, d, g_force_big)));
  part = std::max(part, pf_partial_floats(pf_plan(M, d, f, g_force_big)));
  char *W;
  bf16_t *Ah, *Al, *Mh, *Ml, *kv;
  float *X, *Q, *AO, *P, *rope, *gain;
  int32_t *ptab;
  CK(hipMalloc(&W, wbytes));
  CK(hipMemset(W, 0x3c, wbytes));                       // bf16 0x3c3c = 0.0115: finite products
  CK(hipMalloc(&Ah, 2 * (size_t)mpad * kmax));
  CK(hipMalloc(&Al, 2 * (size_t)mpad * kmax));
  CK(hipMemset(Ah, 0x3c, 2 * (size_t)mpad * kmax));
  CK(hipMemset(Al, 0x38, 2 * (size_t)mpad * kmax));     // 0x3838 = 4.4e-5
  CK(hipMalloc(&Mh, 2 * (size_t)mpad * f));
  CK(hipMalloc(&Ml, 2 * (size_t)mpad * f));
  CK(hipMalloc(&X, 4 * (size_t)mpad * d));
  CK(hipMemset(X, 0, 4 * (size_t)mpad * d));
  CK(hipMalloc(&Q, 4 * (size_t)mpad * nq));
  CK(hipMalloc(&AO, 4 * (size_t)mpad * nq));
  CK(hipMalloc(&P, part ? 4 * part : 256));
  CK(hipMalloc(&gain, 4 * (size_t)d));
  CK(hipMalloc(&rope, 4 * (size_t)mpad * hd));          // cos then sin, [M][hd/2] each
  CK(hipMalloc(&kv, 2 * (size_t)n_pages * n_kv * 2 * pt * hd));
  CK(hipMemset(kv, 0, 2 * (size_t)n_pages * n_kv * 2 * pt * hd));
  CK(hipMalloc(&ptab, 4 * (size_t)n_pages));
  {
    int32_t *h = (int32_t *)malloc(4 * (size_t)n_pages);
    for (int i = 0; i < n_pages; ++i) h[i] = (int)(((long long)i * 7 + 3) % n_pages);      // a permutation when n_pages % 7 != 0
    if (n_pages % 7 == 0) for (int i = 0; i < n_pages; ++i) h[i] = i;
    CK(hipMemcpy(ptab, h, 4 * (size_t)n_pages, hipMemcpyHostToDevice));
    free(h);
  }
  hipLaunchKernelGGL(k_fill_f32, dim3(256), dim3(256), 0, 0, rope, (size_t)mpad * (hd / 2), 0.8f);
  hipLaunchKernelGGL(k_fill_f32, dim3(256), dim3(256), 0, 0, rope + (size_t)mpad * (hd / 2), (size_t)mpad * (hd / 2), 0.6f);
  hipLaunchKernelGGL(k_fill_f32, dim3(16), dim3(256), 0, 0, gain, (size_t)d, 1.0f);
  CK(hipDeviceSynchronize());

  Common c{};
  c.rope_cos = rope;
  c.rope_sin = rope + (size_t)mpad * (hd / 2);
  c.page_table = ptab;
  c.kv_pool = kv;
  c.dm = Dims{};
  c.dm.d = d; c.dm.n_h = n_h; c.dm.n_kv = n_kv; c.dm.hd = hd; c.dm.f = f; c.dm.L = 1; c.dm.E = 1;
  c.dm.max_seq = mpad; c.dm.page_tokens = pt; c.dm.page_shift = 4; c.dm.n_pages = n_pages; c.dm.eps = 1e-5f; c.dm.qscale = 0.0883883f;

  CK(pf_prepare());
  hipEvent_t e0, e1;
  CK(hipEventCreate(&e0));
  CK(hipEventCreate(&e1));
  printf("device: %d CUs; %d positions, d=%d f=%d heads=%d/%d x %d; %d launches each\n", n_cu, M, d, f, n_h, n_kv, hd, iters);

  auto run = [&](const char *name, size_t mat_bytes, double flop, auto launch) {
    const int parts = mat_bytes ? (int)(wbytes / mat_bytes) : 1;
    for (int i = 0; i < 2; ++i) launch((const bf16_t *)(W + (size_t)(i % parts) * mat_bytes));
    (void)hipDeviceSynchronize();
    (void)hipEventRecord(e0);
    for (int i = 0; i < iters; ++i) launch((const bf16_t *)(W + (size_t)((i + 2) % parts) * mat_bytes));
    (void)hipEventRecord(e1);
    (void)hipEventSynchronize(e1);
    float ms = 0.f;
    (void)hipEventElapsedTime(&ms, e0, e1);
    ms /= iters;
    printf("%-24s %8.2f us/launch  %7.1f TFLOP/s algorithmic  %7.1f TFLOP/s on the matrix cores", name, ms * 1e3, flop / ms / 1e9,
           2 * flop / ms / 1e9);
    if (mat_bytes) printf("  weights %6.1f MB -> %5.0f GB/s", mat_bytes / 1e6, mat_bytes / ms / 1e6);
    printf("\n");
    fflush(stdout);
  };
  PfGemm g{};
  g.n_valid = M; g.c0 = 0; g.layer = 0; g.X = X; g.Q = Q; g.Mh = Mh; g.Ml = Ml; g.Ah = Ah; g.Al = Al; g.part = P;
  {
    const PfPlan a = pf_plan(M, qkv_cols, d, g_force_big), b = pf_plan(M, d, nq, g_force_big), u = pf_plan(M, 2 * f, d, g_force_big),
                 w = pf_plan(M, d, f, g_force_big);
    printf("tile edge x K ranges per output tile: qkv %dx%d, o_proj %dx%d, gate_up %dx%d, down %dx%d\n", a.big, a.splits, b.big, b.splits,
           u.big, u.splits, w.big, w.splits);
  }
  run("k_pf_gemm qkv", (size_t)qkv_cols * d * 2, 2.0 * M * qkv_cols * d, [&](const bf16_t *w) {
    PfGemm h = g; h.W = w; h.K = d;
    launch_gemm<kPfQkv>(c, h, qkv_cols);
  });
  run("k_pf_gemm o_proj", (size_t)d * nq * 2, 2.0 * M * d * nq, [&](const bf16_t *w) {
    PfGemm h = g; h.W = w; h.K = nq;
    launch_gemm<kPfResid>(c, h, d);
  });
  run("k_pf_gemm gate_up", (size_t)2 * f * d * 2, 2.0 * M * 2 * f * d, [&](const bf16_t *w) {
    PfGemm h = g; h.W = w; h.K = d;
    launch_gemm<kPfSwiglu>(c, h, 2 * f);
  });
  run("k_pf_gemm down", (size_t)d * f * 2, 2.0 * M * d * f, [&](const bf16_t *w) {
    PfGemm h = g; h.W = w; h.K = f; h.Ah = Mh; h.Al = Ml;
    launch_gemm<kPfResid>(c, h, d);
  });
  run("k_pf_split (norm)", 0, 0.0, [&](const bf16_t *) {
    hipLaunchKernelGGL(k_pf_split, dim3((M + 3) / 4), dim3(kPfBlock), 0, 0, (const float *)X, d, M, (const float *)gain, 1e-5f, Ah, Al);
  });
  CK(hipMemset(Ah, 0x3c, 2 * (size_t)mpad * kmax));
  CK(hipMemset(Al, 0x38, 2 * (size_t)mpad * kmax));
  const int qp = kPfBM / G;
  const dim3 agrid(n_kv, (M + qp - 1) / qp);
  run("k_pf_flash", 0, 2.0 * M * M * hd * n_h, [&](const bf16_t *) {
    if (G == 1) hipLaunchKernelGGL((k_pf_flash<1>), agrid, dim3(kPfBlock), 0, 0, c, 0, 0, M, (const float *)Q, AO);
    else if (G == 2) hipLaunchKernelGGL((k_pf_flash<2>), agrid, dim3(kPfBlock), 0, 0, c, 0, 0, M, (const float *)Q, AO);
    else hipLaunchKernelGGL((k_pf_flash<4>), agrid, dim3(kPfBlock), 0, 0, c, 0, 0, M, (const float *)Q, AO);
  });
  CK(hipGetLastError());
  CK(hipDeviceSynchronize());
  return 0;
}
