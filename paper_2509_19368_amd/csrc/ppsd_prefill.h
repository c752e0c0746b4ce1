// Prefill on the matrix cores: the prompt is processed in chunks of up to kPfChunkMax positions;
// inside a chunk every projection is a dense [positions x K] x [K x N] contraction and runs on MFMA
// (v_mfma_f32_32x32x16_bf16), with the layer's element-wise work fused into the GEMM epilogues
// (rotary + KV append, residual add, SwiGLU).  bf16 storage, head_dim 128.
//
// Precision: weights enter at their stored bf16 values; the fp32 activations are split, once per
// projection input, into a bf16 high part and a bf16 low part (a = hi + lo up to 2^-17 relative)
// and both parts are multiplied, so the products carry fp32-grade activations like the decode
// path's FMA chains, and the accumulators are fp32.  Attention over the chunk's queries is a
// flash-style MFMA kernel of its own (k_pf_flash).
//
// The GEMM comes in two tile shapes.  Small: 128 x 128 outputs per workgroup, 4 waves x (32 positions x
// 128 features), two workgroups per compute unit.  Big: 256 x 256 outputs, 8 waves x (64 positions x
// 128 features), one workgroup per compute unit; it moves half the operand bytes per MFMA through
// L2 and LDS and is taken when it still fills the chip.  K step 32.  LDS holds two stages of
// (A high, A low, W) tiles; a row is 64 bytes and its four 16-byte vectors are stored at position
// v ^ ((row / 4) % 4), which makes both the staging stores (4 rows x 4 vectors per 16 lanes) and the
// MFMA operand loads (16 rows, one vector) hit every bank once.  The next tiles travel in registers
// while the current one is multiplied; one barrier per K step in the small tile, one per half step in
// the big one, whose two halves run half a step apart (see the kernel).  Few output tiles
// (short prompts) are split along K over several workgroups, whose partial tiles a second kernel
// adds in a fixed order before the epilogue, so results do not depend on timing.
// Workgroup ids map to tiles so that all tiles of one weight row block run on one XCD (ids go
// round-robin over the 8 XCDs): each weight tile is fetched from HBM into one L2 only.
#pragma once

#include "ppsd_kernels.h"

namespace ppsd {

constexpr int kPfChunkMax = 4096;   // positions per prefill chunk, at most
constexpr int kPfBM = 128;          // positions per unit tile (4 waves x 32)
constexpr int kPfBN = 128;          // output features per unit tile (4 MFMA tiles of 32)
constexpr int kPfBK = 32;           // K step (2 MFMA k-blocks of 16)
constexpr int kPfBlock = 256;       // threads per unit tile
constexpr int kPfXcds = 8;
constexpr int kPfTargetWgs = 512;   // small tiles: K is split until about this many workgroups exist
constexpr int kPfBigTargetWgs = 256;// big tiles: one per compute unit
constexpr int kPfBigMinTiles = 96;  // big tiles are taken from this many of them on
constexpr int kPfMaxSplit = 8;
constexpr int kPfMinSteps = 4;      // K steps per split, at least

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

enum PfEpilogue : int { kPfQkv = 0, kPfResid = 1, kPfSwiglu = 2 };

// tiles_m, tiles_n count unit tiles (128 x 128); big = 1 or 2 is the workgroup tile's edge in unit tiles.
struct PfPlan { int tiles_m, tiles_n, splits, big; };

// How a [n_valid x n_cols] output with inner length K is cut into workgroups.
// force_big: -1 = choose, 1 / 2 = that tile edge.
inline PfPlan pf_plan(int n_valid, int n_cols, int K, int force_big = -1) {
  PfPlan p;
  p.tiles_m = (n_valid + kPfBM - 1) / kPfBM;
  p.tiles_n = n_cols / kPfBN;
  const int big_tiles = ((p.tiles_m + 1) / 2) * ((p.tiles_n + 1) / 2);
  p.big = force_big > 0 ? force_big : (p.tiles_m >= 2 && big_tiles >= kPfBigMinTiles) ? 2 : 1;
  const int tiles = p.big == 2 ? big_tiles : p.tiles_m * p.tiles_n;
  const int target = p.big == 2 ? kPfBigTargetWgs : kPfTargetWgs, steps = K / kPfBK;
  int s = 1;
  if (tiles < target) s = p.big == 2 ? (target + tiles / 2) / tiles : (target + tiles - 1) / tiles;
  if (s > kPfMaxSplit) s = kPfMaxSplit;
  if (s > steps / kPfMinSteps) s = steps / kPfMinSteps;
  p.splits = s < 1 ? 1 : s;
  return p;
}
// Floats of partial-sum storage the plan needs (0 when K is not split).
inline size_t pf_partial_floats(const PfPlan &p) {
  return p.splits > 1 ? (size_t)p.splits * p.tiles_m * kPfBM * p.tiles_n * kPfBN : 0;
}

struct PfGemm {
  const bf16_t *Ah, *Al; // [chunk][K] high and low parts of the activations
  const bf16_t *W;       // [N_total][K] row-major
  int K;
  int n_valid;           // positions in this chunk
  int c0;                // first position of the chunk
  int layer;
  int tiles_m, tiles_n, splits;   // unit tiles of the output, K ranges
  float *part;           // [splits][tiles_m*128][tiles_n*128] partial sums, when splits > 1
  // epilogue targets
  float *X;              // kPfResid: X[p][n] += C (row pitch d)
  float *Q;              // kPfQkv: rotated queries [chunk][n_h*hd]
  bf16_t *Mh, *Ml;       // kPfSwiglu: [chunk][f], high and low parts
};

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));

// Two floats to packed bf16, round to nearest even (one v_cvt_pk_bf16_f32).
__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
  const f32x2_t v = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}
// (a, b) = hi + lo with both parts bf16; returns the packed pairs.
__device__ __forceinline__ void split_bf16x2(float a, float b, uint32_t &hi, uint32_t &lo) {
  hi = pack_bf16x2(a, b);
  lo = pack_bf16x2(a - __uint_as_float(hi << 16), b - __uint_as_float(hi & 0xffff0000u));
}
__device__ __forceinline__ void split_bf16(float v, bf16_t &hi, bf16_t &lo) {
  uint32_t h, l;
  split_bf16x2(v, 0.f, h, l);
  hi = (bf16_t)h; lo = (bf16_t)l;
}

// hi/lo[p][:] = split(src[p][:] * (gain ? gain[:] / sqrt(mean(src[p]^2) + eps) : 1)); one wave per position.
__global__ __launch_bounds__(kPfBlock) void k_pf_split(const float *src, int K, int n_valid, const float *gain, float eps,
                                                      bf16_t *hi, bf16_t *lo) {
  const int p = blockIdx.x * (kPfBlock / kWave) + (threadIdx.x >> 6);
  if (p >= n_valid) return;
  const int lane = threadIdx.x & 63;
  const float *x = src + (size_t)p * K;
  float rs = 1.0f;
  if (gain) {
    float ss = 0.f;
    for (int i = lane * 4; i < K; i += kWave * 4) {
      const float4 v = *(const float4 *)(x + i);
      ss = fmaf(v.x, v.x, ss); ss = fmaf(v.y, v.y, ss); ss = fmaf(v.z, v.z, ss); ss = fmaf(v.w, v.w, ss);
    }
    ss = wave_sum(ss);
    rs = 1.0f / sqrtf(ss / (float)K + eps);
  }
  for (int i = lane * 4; i < K; i += kWave * 4) {
    float4 v = *(const float4 *)(x + i);
    if (gain) {
      const float4 gg = *(const float4 *)(gain + i);
      v.x *= rs * gg.x; v.y *= rs * gg.y; v.z *= rs * gg.z; v.w *= rs * gg.w;
    }
    uint2 h, l;
    split_bf16x2(v.x, v.y, h.x, l.x);
    split_bf16x2(v.z, v.w, h.y, l.y);
    *(uint2 *)(hi + (size_t)p * K + i) = h;
    *(uint2 *)(lo + (size_t)p * K + i) = l;
  }
}

// X[p][:] = Emb[prompt[c0 + p]][:] as fp32.
__global__ __launch_bounds__(kPfBlock) void k_pf_embed(const bf16_t *embed, const int32_t *prompt, int c0, int n_valid, int d,
                                                      float *X) {
  const int p = blockIdx.x;
  if (p >= n_valid) return;
  const bf16_t *row = embed + (size_t)prompt[c0 + p] * d;
  for (int i = threadIdx.x * 4; i < d; i += kPfBlock * 4) *(float4 *)(X + (size_t)p * d + i) = load4_as_float(row + i);
}

// What happens to the four values v[nt] = C[p][tile column nt*32 + col] of one output tile row.
// Tile column r is weight row:  plain: tile_n*128 + r;  kPfSwiglu: r < 64 -> gate row tile_n*64 + r,
// else up row f + tile_n*64 + (r - 64), so that gate_i sits in v[nt] and up_i in v[nt + 2], exactly
// like the rotary pair (i, i + 64) of a head in kPfQkv.
template <int EPI>
__device__ __forceinline__ void pf_epilogue(const Common &c, const PfGemm &g, int tile_n, int p, int col, const float (&v)[4]) {
  const Dims &m = c.dm;
  if (EPI == kPfResid) {
    float *xr = g.X + (size_t)p * m.d + tile_n * kPfBN + col;
#pragma unroll
    for (int nt = 0; nt < 4; ++nt) xr[nt * 32] += v[nt];
  } else if (EPI == kPfSwiglu) {
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
      const float gt = v[nt], up = v[nt + 2];
      const size_t at = (size_t)p * m.f + tile_n * 64 + nt * 32 + col;
      split_bf16(gt / (1.0f + __expf(-gt)) * up, g.Mh[at], g.Ml[at]);
    }
  } else {   // kPfQkv: tile_n is the head
    const int h = tile_n, pos = g.c0 + p, half = m.hd >> 1;
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
      const int i = nt * 32 + col;
      float lo = v[nt], hi = v[nt + 2];
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

struct PfRegs { uint4 ah0, ah1, al0, al1, w0, w1; };   // one K step of the three tiles, this thread's share

// Element offset of the 16-byte vector v (8 consecutive k) of tile row r inside one LDS plane.
__device__ __forceinline__ int pf_lds_at(int r, int v) { return (r * 4 + (v ^ ((r >> 2) & 3))) * 8; }

// One BIG*128 x BIG*128 output tile (or one K range of it) per workgroup of BIG*256 threads; 1-D grid of
// 8 * ceil(tiles_m / BIG) * splits * ceil(ceil(tiles_n / BIG) / 8) workgroups; BIG * 48 KB of dynamic LDS.
template <int EPI, int BIG>
__global__ __launch_bounds__(kPfBlock *BIG) void k_pf_gemm(Common c, PfGemm g) {
  constexpr int ROWS = 128 * BIG, PLANE = ROWS * kPfBK, STAGE = 3 * PLANE, HALF = ROWS / 2;
  extern __shared__ __attribute__((aligned(16))) bf16_t pf_lds[];   // [2 stages][A high, A low, W][ROWS][32]
  const Dims &m = c.dm;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, wm = wave & 3, wn = wave >> 2;
  const int gm = (g.tiles_m + BIG - 1) / BIG, gn = (g.tiles_n + BIG - 1) / BIG;
  // id -> (XCD, then position tile fastest, then K range, then weight row block)
  const int xcd = blockIdx.x % kPfXcds, local = blockIdx.x / kPfXcds;
  const int tile_m = local % gm, rest = local / gm;
  const int split = rest % g.splits, tile_n = (rest / g.splits) * kPfXcds + xcd;
  if (tile_n >= gn) return;
  const int K = g.K, steps = K / kPfBK;
  const int step0 = (int)((long long)steps * split / g.splits), nk = (int)((long long)steps * (split + 1) / g.splits) - step0;

  // staging: thread t moves, per tile, the 16-byte vector (t % 4) of rows t/4 and t/4 + ROWS/2
  const int srow = tid >> 2, svec = tid & 3;
  const int prow0 = min(tile_m * ROWS + srow, g.n_valid - 1), prow1 = min(tile_m * ROWS + srow + HALF, g.n_valid - 1);   // clamped
  auto weight_row = [&](int r) {       // tile row r -> row of W; a unit tile beyond the last one repeats the first
    int tn = tile_n * BIG + r / 128;
    if (tn >= g.tiles_n) tn = tile_n * BIG;
    const int rr = r % 128;
    if (EPI == kPfSwiglu) return rr < 64 ? tn * 64 + rr : m.f + tn * 64 + (rr - 64);
    return tn * kPfBN + rr;
  };
  const size_t koff = (size_t)step0 * kPfBK + svec * 8;
  const bf16_t *ah_src0 = g.Ah + (size_t)prow0 * K + koff, *ah_src1 = g.Ah + (size_t)prow1 * K + koff;
  const bf16_t *al_src0 = g.Al + (size_t)prow0 * K + koff, *al_src1 = g.Al + (size_t)prow1 * K + koff;
  const bf16_t *w_src0 = g.W + (size_t)weight_row(srow) * K + koff, *w_src1 = g.W + (size_t)weight_row(srow + HALF) * K + koff;
  auto gload = [&](int kt) {
    const int off = kt * kPfBK;
    PfRegs r;
    r.ah0 = *(const uint4 *)(ah_src0 + off); r.ah1 = *(const uint4 *)(ah_src1 + off);
    r.al0 = *(const uint4 *)(al_src0 + off); r.al1 = *(const uint4 *)(al_src1 + off);
    r.w0 = *(const uint4 *)(w_src0 + off); r.w1 = *(const uint4 *)(w_src1 + off);
    return r;
  };
  const int s_at0 = pf_lds_at(srow, svec), s_at1 = pf_lds_at(srow + HALF, svec);
  auto lstore = [&](const PfRegs r, int st) {
    bf16_t *base = pf_lds + st * STAGE;
    *(uint4 *)(base + s_at0) = r.ah0; *(uint4 *)(base + s_at1) = r.ah1;
    *(uint4 *)(base + PLANE + s_at0) = r.al0; *(uint4 *)(base + PLANE + s_at1) = r.al1;
    *(uint4 *)(base + 2 * PLANE + s_at0) = r.w0; *(uint4 *)(base + 2 * PLANE + s_at1) = r.w1;
  };

  f32x16_t acc[BIG][4];
#pragma unroll
  for (int j = 0; j < BIG; ++j)
#pragma unroll
    for (int nt = 0; nt < 4; ++nt)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[j][nt][v] = 0.f;

  // MFMA operand of a lane: row lane % 32 of a 32-row block, 8 consecutive k at 8 * (lane / 32).  Block
  // bases are multiples of 32, so the row's swizzle term depends on the lane only.
  const int half = lane >> 5, swz = (lane >> 2) & 3;
  const int a_row = (wm * BIG * 32 + (lane & 31)) * kPfBK, b_row = (wn * 128 + (lane & 31)) * kPfBK;
  // A K step = fetch (the step's MFMA operands from LDS into registers, all requested at once: the reads
  // return in order, so the first MFMAs can start while the rest arrive) + mma (the MFMAs, from registers).
  bf16x8_t ah[2][BIG], al[2][BIG], b[2][4];
  auto fetch = [&](int st) {
    const bf16_t *base = pf_lds + st * STAGE;
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
      const int kv = ((kk * 2 + half) ^ swz) * 8;
#pragma unroll
      for (int j = 0; j < BIG; ++j) ah[kk][j] = *(const bf16x8_t *)(base + a_row + j * 32 * kPfBK + kv);
#pragma unroll
      for (int nt = 0; nt < 4; ++nt) b[kk][nt] = *(const bf16x8_t *)(base + 2 * PLANE + b_row + nt * 32 * kPfBK + kv);
#pragma unroll
      for (int j = 0; j < BIG; ++j) al[kk][j] = *(const bf16x8_t *)(base + PLANE + a_row + j * 32 * kPfBK + kv);
    }
  };
  auto mma = [&]() {
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
#pragma unroll
      for (int j = 0; j < BIG; ++j)
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) acc[j][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[kk][j], b[kk][nt], acc[j][nt], 0, 0, 0);
#pragma unroll
      for (int j = 0; j < BIG; ++j)
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) acc[j][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al[kk][j], b[kk][nt], acc[j][nt], 0, 0, 0);
    }
  };
  auto compute = [&](int st) {
    fetch(st);
    mma();
    __builtin_amdgcn_sched_group_barrier(0x100, 2 * (2 * BIG + 4), 0);   // the LDS reads, all of them
    __builtin_amdgcn_sched_group_barrier(0x008, 2 * 2 * BIG * 4, 0);     // then the MFMAs
  };

  // Stage kt % 2 holds K step kt.  Load indices are clamped to the last step: the surplus loads and
  // stores at the end touch valid memory and are never read.  The scheduling fences keep the order written.
  if constexpr (BIG == 2) {
    // Two waves share a SIMD (waves w and w + 4).  Running in step they would fetch together and leave the
    // matrix cores idle meanwhile, so the two halves of the workgroup run half a step apart: while waves
    // 0-3 multiply step kt, waves 4-7 do their memory phase of step kt (operands of step kt from LDS
    // into registers, the global tile kt + 1 from registers into the other LDS stage, the request for tile
    // kt + 2); then they swap.  One barrier per half step.  Tile kt + 1 is complete in LDS after both
    // halves' memory phases of step kt and is first read in a memory phase of step kt + 1, behind a barrier;
    // the stage it overwrites was last read in the memory phases of step kt - 1, also behind a barrier.
    const bool ahead = wave < 4;      // waves w and w + 4 share a SIMD (measured: other pairings run 1.4x slower)
    PfRegs r = gload(0);
    lstore(r, 0);
    r = gload(min(1, nk - 1));
    __syncthreads();
    auto memory_phase = [&](int kt) {
      fetch(kt & 1);
      lstore(r, (kt + 1) & 1);
      r = gload(min(kt + 2, nk - 1));
    };
    if (ahead) memory_phase(0);
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
      if (ahead) mma(); else memory_phase(kt);
      __syncthreads();
      if (!ahead) mma(); else if (kt + 1 < nk) memory_phase(kt + 1);
      __syncthreads();
    }
  } else {
    // Steps are short (16 MFMAs per wave) and K ranges too: two register sets, a load has two steps to arrive.
    PfRegs r0 = gload(0), r1 = gload(min(1, nk - 1));
    lstore(r0, 0);
    __syncthreads();
    for (int kt = 0; kt + 2 <= nk; kt += 2) {
      r0 = gload(min(kt + 2, nk - 1));
      __builtin_amdgcn_sched_barrier(0);
      compute(0);
      __builtin_amdgcn_sched_barrier(0);
      lstore(r1, 1);
      __syncthreads();
      r1 = gload(min(kt + 3, nk - 1));
      __builtin_amdgcn_sched_barrier(0);
      compute(1);
      __builtin_amdgcn_sched_barrier(0);
      lstore(r0, 0);
      __syncthreads();
    }
    if (nk & 1) compute(0);
  }


  // acc[j][nt][v]: row wm*BIG*32 + j*32 + 8*(v/4) + 4*(lane/32) + v%4 of the workgroup tile, column nt*32 + lane%32
  // of unit tile tn
  const int tn = tile_n * BIG + wn;
  if (tn >= g.tiles_n) return;
  const int col = lane & 31;
  const size_t ncols = (size_t)g.tiles_n * kPfBN, mpad = (size_t)g.tiles_m * kPfBM;
#pragma unroll
  for (int j = 0; j < BIG; ++j)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int p = tile_m * ROWS + wm * BIG * 32 + j * 32 + 8 * (v >> 2) + 4 * half + (v & 3);
      if (p >= g.n_valid) continue;
      if (g.splits > 1) {
        float *dst = g.part + ((size_t)split * mpad + p) * ncols + (size_t)tn * kPfBN + col;
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) dst[nt * 32] = acc[j][nt][v];
      } else {
        const float vals[4] = {acc[j][0][v], acc[j][1][v], acc[j][2][v], acc[j][3][v]};
        pf_epilogue<EPI>(c, g, tn, p, col, vals);
      }
    }
}

// Adds the K ranges' partial tiles in range order and runs the epilogue; grid (tiles_n, ceil(n_valid / 8)).
template <int EPI>
__global__ __launch_bounds__(kPfBlock) void k_pf_reduce(Common c, PfGemm g) {
  const int tile_n = blockIdx.x, p = blockIdx.y * (kPfBlock / 32) + (threadIdx.x >> 5), col = threadIdx.x & 31;
  if (p >= g.n_valid) return;
  const size_t ncols = (size_t)g.tiles_n * kPfBN, mpad = (size_t)g.tiles_m * kPfBM;
  float v[4] = {0.f, 0.f, 0.f, 0.f};
  for (int s = 0; s < g.splits; ++s) {
    const float *src = g.part + ((size_t)s * mpad + p) * ncols + (size_t)tile_n * kPfBN + col;
#pragma unroll
    for (int nt = 0; nt < 4; ++nt) v[nt] += src[nt * 32];
  }
  pf_epilogue<EPI>(c, g, tile_n, p, col, v);
}

// Dynamic LDS of the big-tile GEMM exceeds the default limit: raise it once per process and device.
template <int EPI>
inline hipError_t pf_allow_big_lds() {
  return hipFuncSetAttribute((const void *)k_pf_gemm<EPI, 2>, hipFuncAttributeMaxDynamicSharedMemorySize, 2 * 3 * 256 * kPfBK * 2);
}
inline hipError_t pf_prepare() {
  hipError_t e = pf_allow_big_lds<kPfQkv>();
  if (e == hipSuccess) e = pf_allow_big_lds<kPfResid>();
  if (e == hipSuccess) e = pf_allow_big_lds<kPfSwiglu>();
  return e;
}

// One projection of a chunk: the GEMM over g.n_valid positions and n_cols output columns, then, when K
// was split, the kernel that adds the partial tiles and runs the epilogue.  g.part must hold
// pf_partial_floats(pl) floats.
template <int EPI>
inline void pf_launch(hipStream_t stream, const Common &c, PfGemm g, const PfPlan &pl) {
  g.tiles_m = pl.tiles_m; g.tiles_n = pl.tiles_n; g.splits = pl.splits;
  const int gm = (pl.tiles_m + pl.big - 1) / pl.big, gn = (pl.tiles_n + pl.big - 1) / pl.big;
  const dim3 grid(kPfXcds * gm * pl.splits * ((gn + kPfXcds - 1) / kPfXcds));
  const size_t lds = (size_t)pl.big * 2 * 3 * 128 * kPfBK * 2;
  if (pl.big == 2) hipLaunchKernelGGL((k_pf_gemm<EPI, 2>), grid, dim3(2 * kPfBlock), lds, stream, c, g);
  else hipLaunchKernelGGL((k_pf_gemm<EPI, 1>), grid, dim3(kPfBlock), lds, stream, c, g);
  if (pl.splits > 1)
    hipLaunchKernelGGL((k_pf_reduce<EPI>), dim3(pl.tiles_n, (g.n_valid + kPfBlock / 32 - 1) / (kPfBlock / 32)), dim3(kPfBlock), 0,
                       stream, c, g);
}

// Attention of the chunk's queries on the matrix cores (causal, online softmax over tiles of 32 keys).
// A workgroup takes one KV head and 128 query rows that share it: G query heads x 128/G consecutive
// positions, 32 rows per wave.  Per key tile a wave forms S^T = K Q^T (keys as MFMA rows, its 32 queries as
// columns), so a lane owns one query and 16 of the tile's 32 keys: maximum and sum are in-lane plus one
// exchange with lane + 32, the rescaling factor is a per-lane scalar, and the probabilities leave the
// accumulator already in the layout of the next MFMA's B operand.  O^T += V^T P^T then wants, per lane,
// 8 keys of one feature: the V tile is written to LDS transposed, keys in the order the accumulator
// holds them (bits 2 and 3 of the key index swapped).  K and V are stored bf16 and enter exactly; the fp32
// queries (pre-scaled by 1/sqrt(hd)) and the probabilities are split into bf16 high + low parts and both
// are multiplied, as in the GEMMs.  LDS holds two stages of (K, V^T); the next tiles travel in registers.
constexpr int kFaKeys = 32;
constexpr int kFaKPitch = 128 + 8;       // K tile row pitch in bf16 elements (272 bytes)
constexpr int kFaVPitch = kFaKeys + 8;   // V^T tile row pitch (80 bytes)

struct FaRegs { uint4 k0, k1, v0, v1; };

__device__ __forceinline__ int fa_key_column(int key) { return (key & ~12) | ((key & 4) << 1) | ((key & 8) >> 1); }

__device__ __forceinline__ void fa_split8(const float (&x)[8], bf16x8_t &hi, bf16x8_t &lo) {
  uint4 h, l;
  split_bf16x2(x[0], x[1], h.x, l.x); split_bf16x2(x[2], x[3], h.y, l.y);
  split_bf16x2(x[4], x[5], h.z, l.z); split_bf16x2(x[6], x[7], h.w, l.w);
  hi = __builtin_bit_cast(bf16x8_t, h);
  lo = __builtin_bit_cast(bf16x8_t, l);
}

// grid (n_kv, ceil(n_valid / (128 / G))); Q and AO are [chunk][n_h * 128] fp32.
template <int G>
__global__ __launch_bounds__(kPfBlock, 2) void k_pf_flash(Common c, int layer, int c0, int n_valid, const float *Q, float *AO) {
  constexpr int HD = 128, WPH = 4 / G, QP = 32 * WPH;
  __shared__ __attribute__((aligned(16))) bf16_t sK[2][kFaKeys * kFaKPitch];
  __shared__ __attribute__((aligned(16))) bf16_t sVt[2][HD * kFaVPitch];
  const Dims &m = c.dm;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, half = lane >> 5;
  const int kvh = blockIdx.x;
  const int q0 = ((int)gridDim.y - 1 - (int)blockIdx.y) * QP;        // long key ranges first
  const int pw = q0 + 32 * (wave % WPH), head = kvh * G + wave / WPH;
  const int my_p = pw + (lane & 31);
  const int my_pos = c0 + min(my_p, n_valid - 1);
  const size_t nq = (size_t)m.n_h * HD;
  const int n_keys = c0 + min(q0 + QP, n_valid);                    // keys 0 .. last query position of the workgroup
  const int n_tiles = (n_keys + kFaKeys - 1) / kFaKeys;

  // the lane's query as B operands: feature block kb of 16, features 16*kb + 8*half + 0..7
  bf16x8_t qh[HD / 16], ql[HD / 16];
  {
    const float *qr = Q + (size_t)min(my_p, n_valid - 1) * nq + (size_t)head * HD + 8 * half;
    const float qs = m.qscale * 1.44269504088896341f;       // scores in units of log 2: exp becomes exp2
#pragma unroll
    for (int kb = 0; kb < HD / 16; ++kb) {
      const float4 a = *(const float4 *)(qr + 16 * kb), b = *(const float4 *)(qr + 16 * kb + 4);
      const float x[8] = {a.x * qs, a.y * qs, a.z * qs, a.w * qs, b.x * qs, b.y * qs, b.z * qs, b.w * qs};
      fa_split8(x, qh[kb], ql[kb]);
    }
  }

  // staging: K rows tid/16 and tid/16 + 16, 16-byte vector tid%16; V row tid%32, vectors tid/32 and tid/32 + 8
  const int k_key = tid >> 4, k_vec = (tid & 15) * 8, v_key = tid & 31, v_vec = (tid >> 5) * 8;
  auto gload = [&](int kt) {
    FaRegs r;
    const int base = kt * kFaKeys, last = n_keys - 1;
    r.k0 = *(const uint4 *)(kv_row<bf16_t>(c, c.page_table, layer, min(base + k_key, last), kvh, 0) + k_vec);
    r.k1 = *(const uint4 *)(kv_row<bf16_t>(c, c.page_table, layer, min(base + k_key + 16, last), kvh, 0) + k_vec);
    const bf16_t *vr = kv_row<bf16_t>(c, c.page_table, layer, min(base + v_key, last), kvh, 1);
    r.v0 = *(const uint4 *)(vr + v_vec);
    r.v1 = *(const uint4 *)(vr + v_vec + 64);
    return r;
  };
  const int v_col = fa_key_column(v_key);
  auto lstore = [&](const FaRegs r, int st) {
    *(uint4 *)(&sK[st][k_key * kFaKPitch + k_vec]) = r.k0;
    *(uint4 *)(&sK[st][(k_key + 16) * kFaKPitch + k_vec]) = r.k1;
    const uint32_t a[4] = {r.v0.x, r.v0.y, r.v0.z, r.v0.w}, b[4] = {r.v1.x, r.v1.y, r.v1.z, r.v1.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      sVt[st][(v_vec + 2 * e) * kFaVPitch + v_col] = (bf16_t)(a[e] & 0xffffu);
      sVt[st][(v_vec + 2 * e + 1) * kFaVPitch + v_col] = (bf16_t)(a[e] >> 16);
      sVt[st][(v_vec + 64 + 2 * e) * kFaVPitch + v_col] = (bf16_t)(b[e] & 0xffffu);
      sVt[st][(v_vec + 64 + 2 * e + 1) * kFaVPitch + v_col] = (bf16_t)(b[e] >> 16);
    }
  };

  f32x16_t o[HD / 32];                     // O^T: feature 32*dt + 8*(v/4) + 4*half + v%4 of the lane's query
#pragma unroll
  for (int dt = 0; dt < HD / 32; ++dt)
#pragma unroll
    for (int v = 0; v < 16; ++v) o[dt][v] = 0.f;
  float mx = -INFINITY, sum = 0.f;         // running maximum; this lane's share of the running sum

  const int ka_at = (lane & 31) * kFaKPitch + 8 * half;     // K as A operand: key lane%32, 8 features
  const int va_at = (lane & 31) * kFaVPitch + 8 * half;     // V^T as A operand: feature lane%32, 8 keys
  auto compute = [&](int kt, int st) {
    if (kt * kFaKeys > c0 + pw + 31) return;                 // every key of the tile lies behind the wave's queries
    f32x16_t s;
#pragma unroll
    for (int v = 0; v < 16; ++v) s[v] = 0.f;
#pragma unroll
    for (int kb = 0; kb < HD / 16; ++kb) {
      const bf16x8_t ka = *(const bf16x8_t *)(&sK[st][ka_at + 16 * kb]);
      s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qh[kb], s, 0, 0, 0);
      s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, ql[kb], s, 0, 0, 0);
    }
    // s[v]: key kt*32 + 8*(v/4) + 4*half + v%4 against the lane's query, in units of log 2
    if (kt * kFaKeys + kFaKeys - 1 > c0 + pw) {              // the tile reaches past the wave's first query: mask
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int key = kt * kFaKeys + 8 * (v >> 2) + 4 * half + (v & 3);
        s[v] = key <= my_pos ? s[v] : -INFINITY;
      }
    }
    float tmax = s[0];
#pragma unroll
    for (int v = 1; v < 16; ++v) tmax = fmaxf(tmax, s[v]);
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
    const float mn = fmaxf(mx, tmax);
    const float corr = __builtin_amdgcn_exp2f(mx - mn);
    mx = mn;
    float p[16], psum = 0.f;
#pragma unroll
    for (int v = 0; v < 16; ++v) { p[v] = __builtin_amdgcn_exp2f(s[v] - mn); psum += p[v]; }
    sum = sum * corr + psum;
    if (__any(corr != 1.0f)) {                               // some query's maximum rose
#pragma unroll
      for (int dt = 0; dt < HD / 32; ++dt)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[dt][v] *= corr;
    }
    bf16x8_t ph[2], pl[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      const float x[8] = {p[8 * kb], p[8 * kb + 1], p[8 * kb + 2], p[8 * kb + 3], p[8 * kb + 4], p[8 * kb + 5], p[8 * kb + 6], p[8 * kb + 7]};
      fa_split8(x, ph[kb], pl[kb]);
    }
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      bf16x8_t va[HD / 32];
#pragma unroll
      for (int dt = 0; dt < HD / 32; ++dt) va[dt] = *(const bf16x8_t *)(&sVt[st][va_at + dt * 32 * kFaVPitch + 16 * kb]);
#pragma unroll
      for (int dt = 0; dt < HD / 32; ++dt) o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[dt], ph[kb], o[dt], 0, 0, 0);
#pragma unroll
      for (int dt = 0; dt < HD / 32; ++dt) o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[dt], pl[kb], o[dt], 0, 0, 0);
    }
  };

  // as in the GEMM: stage kt % 2 holds tile kt, r0 / r1 carry the tiles behind it (indices clamped)
  FaRegs r0 = gload(0), r1 = gload(min(1, n_tiles - 1));
  lstore(r0, 0);
  __syncthreads();
  for (int kt = 0; kt + 2 <= n_tiles; kt += 2) {
    r0 = gload(min(kt + 2, n_tiles - 1));
    __builtin_amdgcn_sched_barrier(0);
    compute(kt, 0);
    __builtin_amdgcn_sched_barrier(0);
    lstore(r1, 1);
    __syncthreads();
    r1 = gload(min(kt + 3, n_tiles - 1));
    __builtin_amdgcn_sched_barrier(0);
    compute(kt + 1, 1);
    __builtin_amdgcn_sched_barrier(0);
    lstore(r0, 0);
    __syncthreads();
  }
  if (n_tiles & 1) compute(n_tiles - 1, 0);

  sum += __shfl_xor(sum, 32);
  if (my_p < n_valid) {
    const float inv = 1.0f / sum;
    float *out = AO + (size_t)my_p * nq + (size_t)head * HD + 4 * half;
#pragma unroll
    for (int dt = 0; dt < HD / 32; ++dt)
#pragma unroll
      for (int q = 0; q < 4; ++q)
        *(float4 *)(out + 32 * dt + 8 * q) = make_float4(o[dt][4 * q] * inv, o[dt][4 * q + 1] * inv, o[dt][4 * q + 2] * inv, o[dt][4 * q + 3] * inv);
  }
}

// The last prompt position's residual row becomes the LM head's input.
__global__ void k_pf_last_row(const float *X, int row, int d, float *dst) {
  for (int i = threadIdx.x + blockIdx.x * blockDim.x; i < d; i += blockDim.x * gridDim.x) dst[i] = X[(size_t)row * d + i];
}

}  // namespace ppsd
