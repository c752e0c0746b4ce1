// Prefill on the matrix cores: the prompt is processed in chunks of kPfChunk positions; inside a
// chunk every projection is a dense [positions x K] x [K x N] contraction and runs on MFMA
// (v_mfma_f32_32x32x8_bf16_1k), with the layer's element-wise work fused into the GEMM epilogues
// (rotary + KV append, residual add, SwiGLU).  bf16 storage, head_dim 128.
//
// Precision: weights enter at their stored bf16 values; the fp32 activations are split on the fly
// into a bf16 high part and a bf16 low part (a = hi + lo up to 2^-17 relative) and both parts are
// multiplied, so the products carry fp32-grade activations like the decode path's FMA chains, and
// the accumulators are fp32.  Decode attention over the chunk's queries reuses attn_unit.
#pragma once

#include "ppsd_kernels.h"

namespace ppsd {

constexpr int kPfChunk = 512;    // positions per prefill chunk
constexpr int kPfBM = 128;       // positions per GEMM tile (4 waves x 32)
constexpr int kPfBN = 128;       // output features per GEMM tile (4 MFMA tiles of 32)
constexpr int kPfBK = 32;        // K step
constexpr int kPfLd = kPfBK + 4; // LDS row pitch in bf16 elements (72 bytes)
constexpr int kPfBlock = 256;

typedef short bf16x4_t __attribute__((ext_vector_type(4)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

enum PfEpilogue : int { kPfQkv = 0, kPfResid = 1, kPfSwiglu = 2 };

struct PfGemm {
  const float *A;        // [chunk][K] fp32 activations
  const float *rs;       // [chunk] 1/sqrt(mean(x^2)+eps) per position, or nullptr (no norm)
  const float *gain;     // [K] norm gain, with rs
  const bf16_t *W;       // [N_total][K] row-major
  int K;
  int n_valid;           // positions in this chunk
  int c0;                // first position of the chunk
  int layer;
  // epilogue targets
  float *X;              // kPfResid: X[p][n] += C (row pitch d)
  float *Q;              // kPfQkv: rotated queries [chunk][n_h*hd]
  float *M;              // kPfSwiglu: [chunk][f]
};

// rs[p] = 1/sqrt(mean(X[p]^2) + eps); one wave per position.
__global__ __launch_bounds__(kPfBlock) void k_pf_rowscale(const float *X, int d, int n_valid, float eps, float *rs) {
  const int p = blockIdx.x * (kPfBlock / kWave) + (threadIdx.x >> 6);
  if (p >= n_valid) return;
  const int lane = threadIdx.x & 63;
  const float *x = X + (size_t)p * d;
  float ss = 0.f;
  for (int i = lane * 4; i < d; i += kWave * 4) {
    const float4 v = *(const float4 *)(x + i);
    ss = fmaf(v.x, v.x, ss); ss = fmaf(v.y, v.y, ss); ss = fmaf(v.z, v.z, ss); ss = fmaf(v.w, v.w, ss);
  }
  ss = wave_sum(ss);
  if (lane == 0) rs[p] = 1.0f / sqrtf(ss / (float)d + eps);
}

// X[p][:] = Emb[prompt[c0 + p]][:] as fp32.
__global__ __launch_bounds__(kPfBlock) void k_pf_embed(const bf16_t *embed, const int32_t *prompt, int c0, int n_valid, int d,
                                                      float *X) {
  const int p = blockIdx.x;
  if (p >= n_valid) return;
  const bf16_t *row = embed + (size_t)prompt[c0 + p] * d;
  for (int i = threadIdx.x * 4; i < d; i += kPfBlock * 4) *(float4 *)(X + (size_t)p * d + i) = load4_as_float(row + i);
}

// One 128 x 128 output tile per workgroup.  grid = (N tiles, position tiles).
// Tile row r of the weight operand is W row:  plain: tile_n*128 + r;
// kPfSwiglu: r < 64 -> gate row tile_n*64 + r, else up row f + tile_n*64 + (r - 64), so that a
// lane finds gate_i in MFMA tile j and up_i in tile j + 2, exactly like the rotary pair (i, i + 64).
template <int EPI>
__global__ __launch_bounds__(kPfBlock) void k_pf_gemm(Common c, PfGemm g) {
  __shared__ __attribute__((aligned(16))) bf16_t sAh[kPfBM * kPfLd];
  __shared__ __attribute__((aligned(16))) bf16_t sAl[kPfBM * kPfLd];
  __shared__ __attribute__((aligned(16))) bf16_t sW[kPfBN * kPfLd];
  const Dims &m = c.dm;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int tile_n = blockIdx.x, tile_m = blockIdx.y;
  const int K = g.K;

  // staging assignment: thread t handles tile row t/2, 16 consecutive k at (t%2)*16
  const int srow = tid >> 1, scol = (tid & 1) * 16;
  const int prow = min(tile_m * kPfBM + srow, g.n_valid - 1);            // clamped position row
  const float *a_src = g.A + (size_t)prow * K + scol;
  const float a_rs = g.rs ? g.rs[prow] : 1.0f;
  int wrow;
  if (EPI == kPfSwiglu) wrow = srow < 64 ? tile_n * 64 + srow : m.f + tile_n * 64 + (srow - 64);
  else wrow = tile_n * kPfBN + srow;
  const bf16_t *w_src = g.W + (size_t)wrow * K + scol;

  f32x16_t acc[4];
#pragma unroll
  for (int nt = 0; nt < 4; ++nt)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[nt][v] = 0.f;

  const int a_row = wave * 32 + (lane & 31);   // A-operand row of this lane inside the tile
  const int kq = 4 * (lane >> 5);              // k offset of this lane inside an MFMA k-block of 8

  for (int k0 = 0; k0 < K; k0 += kPfBK) {
    // ---- global -> registers
    float4 av[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) av[e] = *(const float4 *)(a_src + k0 + 4 * e);
    const uint4 w0 = *(const uint4 *)(w_src + k0);
    const uint4 w1 = *(const uint4 *)(w_src + k0 + 8);
    if (g.rs) {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float4 gg = *(const float4 *)(g.gain + k0 + scol + 4 * e);
        av[e].x *= a_rs * gg.x; av[e].y *= a_rs * gg.y; av[e].z *= a_rs * gg.z; av[e].w *= a_rs * gg.w;
      }
    }
    __syncthreads();   // previous step's MFMA reads are done
    // ---- registers -> LDS (activation split into bf16 high and low parts)
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float vals[4] = {av[e].x, av[e].y, av[e].z, av[e].w};
      bf16_t hi[4], lo[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        hi[q] = float_to_bf16_rne(vals[q]);
        lo[q] = float_to_bf16_rne(vals[q] - Pack<bf16_t>::to_float(hi[q]));
      }
      *(uint2 *)(sAh + srow * kPfLd + scol + 4 * e) = make_uint2((uint32_t)hi[0] | ((uint32_t)hi[1] << 16), (uint32_t)hi[2] | ((uint32_t)hi[3] << 16));
      *(uint2 *)(sAl + srow * kPfLd + scol + 4 * e) = make_uint2((uint32_t)lo[0] | ((uint32_t)lo[1] << 16), (uint32_t)lo[2] | ((uint32_t)lo[3] << 16));
    }
    *(uint2 *)(sW + srow * kPfLd + scol) = make_uint2(w0.x, w0.y);
    *(uint2 *)(sW + srow * kPfLd + scol + 4) = make_uint2(w0.z, w0.w);
    *(uint2 *)(sW + srow * kPfLd + scol + 8) = make_uint2(w1.x, w1.y);
    *(uint2 *)(sW + srow * kPfLd + scol + 12) = make_uint2(w1.z, w1.w);
    __syncthreads();
    // ---- MFMA over the K step
#pragma unroll
    for (int kk = 0; kk < kPfBK / 8; ++kk) {
      const bf16x4_t ah = *(const bf16x4_t *)(sAh + a_row * kPfLd + kk * 8 + kq);
      const bf16x4_t al = *(const bf16x4_t *)(sAl + a_row * kPfLd + kk * 8 + kq);
#pragma unroll
      for (int nt = 0; nt < 4; ++nt) {
        const bf16x4_t b = *(const bf16x4_t *)(sW + (nt * 32 + (lane & 31)) * kPfLd + kk * 8 + kq);
        acc[nt] = __builtin_amdgcn_mfma_f32_32x32x8bf16_1k(ah, b, acc[nt], 0, 0, 0);
        acc[nt] = __builtin_amdgcn_mfma_f32_32x32x8bf16_1k(al, b, acc[nt], 0, 0, 0);
      }
    }
  }

  // ---- epilogue.  acc[nt][v]: tile row wave*32 + 8*(v/4) + 4*(lane/32) + v%4, tile column nt*32 + lane%32
  const int col = lane & 31;
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int p = tile_m * kPfBM + wave * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
    if (p >= g.n_valid) continue;
    if (EPI == kPfResid) {
      float *xr = g.X + (size_t)p * m.d + tile_n * kPfBN;
#pragma unroll
      for (int nt = 0; nt < 4; ++nt) xr[nt * 32 + col] += acc[nt][v];
    } else if (EPI == kPfSwiglu) {
#pragma unroll
      for (int nt = 0; nt < 2; ++nt) {
        const float gt = acc[nt][v], up = acc[nt + 2][v];
        g.M[(size_t)p * m.f + tile_n * 64 + nt * 32 + col] = gt / (1.0f + __expf(-gt)) * up;
      }
    } else {   // kPfQkv: tile_n is the head; rotation pair (i, i + 64) = MFMA tiles (nt, nt + 2)
      const int h = tile_n, pos = g.c0 + p, half = m.hd >> 1;
#pragma unroll
      for (int nt = 0; nt < 2; ++nt) {
        const int i = nt * 32 + col;
        float lo = acc[nt][v], hi = acc[nt + 2][v];
        if (h < m.n_h + m.n_kv) {
          const float cs = c.rope_cos[(size_t)pos * half + i], sn = c.rope_sin[(size_t)pos * half + i];
          const float rlo = lo * cs - hi * sn, rhi = hi * cs + lo * sn;
          lo = rlo; hi = rhi;
        }
        if (h < m.n_h) {
          float *qr = g.Q + (size_t)p * (m.n_h * m.hd) + h * m.hd;
          qr[i] = lo; qr[i + half] = hi;
        } else {
          const int which = (h < m.n_h + m.n_kv) ? 0 : 1;
          const int kvh = which ? h - m.n_h - m.n_kv : h - m.n_h;
          bf16_t *dst = kv_row<bf16_t>(c, c.page_table, g.layer, pos, kvh, which);
          dst[i] = float_to_bf16_rne(lo); dst[i + half] = float_to_bf16_rne(hi);
        }
      }
    }
  }
}

// Attention of the chunk's queries: one workgroup per (KV head, query position), keys 0..position.
template <int G>
__global__ __launch_bounds__(kPfBlock) void k_pf_attn(Common c, int layer, int c0, const float *Q, float *AO) {
  constexpr int HD = 128;
  constexpr int GPB = kPfBlock / (HD / Pack<bf16_t>::N);
  __shared__ float merge[GPB * G * (HD + 2)];
  __shared__ int s_last;
  const int p = blockIdx.y;
  const size_t nq = (size_t)c.dm.n_h * HD;
  attn_unit<bf16_t, HD, G, kPfBlock>(c, c.page_table, layer, c0 + p, blockIdx.x, 0, 1, Q + p * nq, AO + p * nq, nullptr,
                                     nullptr, merge, &s_last);
}

// The last prompt position's residual row becomes the LM head's input.
__global__ void k_pf_last_row(const float *X, int row, int d, float *dst) {
  for (int i = threadIdx.x + blockIdx.x * blockDim.x; i < d; i += blockDim.x * gridDim.x) dst[i] = X[(size_t)row * d + i];
}

}  // namespace ppsd
