// Device-side definitions shared by the decode kernels (gfx950, wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ppsd {

typedef uint16_t bf16_t;   // raw bfloat16 bits

constexpr int kWave = 64;
constexpr int kBlock = 256;          // threads per workgroup in every kernel
constexpr int kWavesPerBlock = kBlock / kWave;
constexpr int kGBlock = 512;         // threads per workgroup of the weight-streaming kernels
constexpr int kGWaves = kGBlock / kWave;
constexpr int kTripRows = 2;         // rows a wave streams at a time (one rotation / gate-up pair)
constexpr int kTripBlocks = 2;       // column blocks per trip: 4 independent 16-byte loads per lane.
                                     // Measured on gfx950: many waves with a shallow queue each
                                     // (2 x 2) stream faster than fewer waves with deep queues.
constexpr float kNegBig = -1.0e30f;  // finite stand-in for -inf in the running softmax maximum

// Stage roles: which part of the device state a kernel takes its input from.
// kPipeStage0 + k is stage k of the full ceil(N/E)-stage schedule (Sec. 4.1, Alg. 1).
// kEesdDraft0 + j is draft step j of a draft-then-verify round (Sec. 3.1), kEesdVerify its batched
// verify pass.
enum Role : int { kVanilla = 0, kDraft = 1, kVerify = 2, kPrefill = 3, kPipeStage0 = 16, kEesdDraft0 = 40,
                  kEesdVerify = 48 };

constexpr int kMaxStages = 16;       // stages of the full pipeline schedule
constexpr int kTokRing = 32;         // ring of the tokens stage 0 used, by position (> kMaxStages)

// Residual-stream slots inside xbuf (each d floats).  The two-stage path uses the first four.
// The full pipeline adds one working slot per stage (kXStageWork0 + k, fixed address) and, for the
// boundary in front of stage b >= 1, two buffers that swap roles every tick: the stage reads
// kXBoundRead0 + b while stage b-1 writes kXBoundWrite0 + b.
// Draft-then-verify rounds reuse the boundary buffers' slots: kXBatchIn0 + b holds the layer-E
// hidden state of the round's token b, kXBatchWork0 + b its residual stream in the verify pass.
enum XSel : int { kXDraft = 0, kXVerify = 1, kHExitCur = 2, kHExitNext = 3,
                  kXStageWork0 = 4, kXBoundRead0 = 32, kXBoundWrite0 = 64, kXBatchIn0 = 96, kXBatchWork0 = 112 };
constexpr int kXBatchInSlot0 = 4 + kMaxStages;        // slot index of kXBatchIn0
constexpr int kXBatchWorkSlot0 = kXBatchInSlot0 + 8;  // slot index of kXBatchWork0
constexpr int kXSlots = 4 + kMaxStages + 2 * kMaxStages;   // slots in xbuf

// Device-resident decode state.  Only the commit kernel writes it, once per step, after
// both stages have finished; every other kernel of the step reads a stable copy.
struct DevState {
  int32_t t;            // position of the last committed token
  int32_t last_token;   // y_t
  int32_t full;         // 1: h_t^E and draft d_{t+1} are in hand (pipeline full)
  int32_t draft;        // d_{t+1} when full
  int32_t cur;          // which hExit buffer holds h_t^E when full
  int32_t n_out;        // tokens written to out_tokens by the current decode call
  int32_t target;       // the current decode call stops at n_out == target
  int32_t gen_count;    // tokens committed since prefill, token #0 included
  int32_t prefill_pos;  // next prompt position to process
  int32_t prefill_len;
  int32_t pad[6];
  int64_t stats[12];    // committed, compared, accepted, rejected, overlapped, draft_only, rollbacks, spare,
                        // pipeline ticks, stage runs, flushed in-flight tokens
  // full pipeline schedule: what each stage works on in the coming tick
  int32_t pl_valid[kMaxStages];   // stage k has an input
  int32_t pl_pos[kMaxStages];     // the position it belongs to
  int32_t pl_tok0;                // token stage 0 embeds
  int32_t pl_par;                 // which buffer of every stage boundary is the readable one
  int32_t pl_pad[2];
  int32_t pl_tok_at[kTokRing];    // token stage 0 used at position p, at index p % kTokRing
  // draft-then-verify round: ee_draft[j] = token of draft step j (j >= 1; step 0 takes last_token)
  int32_t ee_draft[8];
};

struct Dims {
  int32_t d, n_h, n_kv, hd, f, V, L, E;
  int32_t max_seq, page_tokens, n_pages, n_splits;
  int32_t debug_rows, head_blocks;
  int32_t n_stages, page_shift;   // ceil(L / E); log2(page_tokens) (pages hold 8, 16, 32 or 64 positions)
  int32_t draft_share;            // of 256: workgroups of a draft-stage kernel that work while the verify stage runs beside it
  float eps, qscale;     // qscale = 1/sqrt(hd)
};

// Everything a kernel needs besides its own operands; passed by value.
struct Common {
  DevState *st;
  const int32_t *prompt;      // [max_seq] prompt ids (device)
  float *xbuf;                // [kXSlots][d]
  const float *rope_cos;      // [max_seq][hd/2]
  const float *rope_sin;
  const int32_t *page_table;  // [n_pages]
  void *kv_pool;              // [L][n_pages][n_kv][2][page_tokens][hd] storage dtype
  Dims dm;
};

struct StageIn {
  int active;
  int pos;
  int tok;
};

// Step a0 of the decode path: which token/position each stage works on.
__device__ __forceinline__ StageIn stage_in(const Common &c, int role) {
  const DevState *st = c.st;
  StageIn s;
  const int running = st->n_out < st->target;
  if (role == kPrefill) {
    s.active = st->prefill_pos < st->prefill_len;
    s.pos = st->prefill_pos;
    s.tok = s.active ? c.prompt[s.pos] : 0;
  } else if (role == kVanilla) {
    s.active = running;
    s.pos = st->t;
    s.tok = st->last_token;
  } else if (role == kDraft) {
    s.active = running;
    s.pos = st->full ? st->t + 1 : st->t;
    s.tok = st->full ? st->draft : st->last_token;
  } else if (role == kVerify) {
    s.active = running && st->full;
    s.pos = st->t;
    s.tok = -1;
  } else if (role >= kEesdDraft0) {
    const int j = (role - kEesdDraft0) & 7;      // kEesdVerify: j = 0, the pass starts at the committed token
    s.active = running;
    s.pos = st->t + (role == kEesdVerify ? 0 : j);
    s.tok = (role == kEesdVerify || j == 0) ? st->last_token : st->ee_draft[j];
  } else {  // kPipeStage0 + k, k < kMaxStages (the host launches no other role)
    const int k = (role - kPipeStage0) & (kMaxStages - 1);
    s.active = running && st->pl_valid[k];
    s.pos = st->pl_pos[k];
    s.tok = k == 0 ? st->pl_tok0 : -1;
  }
  return s;
}

__device__ __forceinline__ float *xslot(const Common &c, int sel) {
  int slot = sel;
  if (sel == kHExitCur) slot = 2 + (c.st->cur & 1);
  else if (sel == kHExitNext) slot = 2 + ((c.st->cur & 1) ^ 1);
  else if (sel >= kXBatchWork0) slot = kXBatchWorkSlot0 + ((sel - kXBatchWork0) & 7);
  else if (sel >= kXBatchIn0) slot = kXBatchInSlot0 + ((sel - kXBatchIn0) & 7);
  else if (sel >= kXBoundWrite0) slot = kXStageWork0 + kMaxStages + 2 * ((sel - kXBoundWrite0) & (kMaxStages - 1)) + ((c.st->pl_par & 1) ^ 1);
  else if (sel >= kXBoundRead0) slot = kXStageWork0 + kMaxStages + 2 * ((sel - kXBoundRead0) & (kMaxStages - 1)) + (c.st->pl_par & 1);
  return c.xbuf + (size_t)slot * c.dm.d;
}

// 16-byte streaming load (weights and probe data are read once per step: keep them out of the
// way of the small, reused activation vectors in the caches).
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 ld16_stream(const void *p) {
  const u32x4_t v = __builtin_nontemporal_load((const u32x4_t *)p);
  return make_uint4(v.x, v.y, v.z, v.w);
}

// Same, for a wave-uniform base pointer known to be global memory plus a per-lane byte offset:
// compiles to a global (not flat) load with a scalar base.
typedef const u32x4_t __attribute__((address_space(1))) *gptr16_t;
__device__ __forceinline__ uint4 ld16_stream_global(const void *base, uint32_t byte_off) {
  const u32x4_t v = __builtin_nontemporal_load((gptr16_t)((uintptr_t)base + byte_off));
  return make_uint4(v.x, v.y, v.z, v.w);
}

// Hand-over of a few values between workgroups that are running at the same time (they may sit
// on different L2 slices, which are not coherent with each other): relaxed atomic accesses at
// agent scope go past the local L2, so no cache-wide write-back or invalidate is needed.  The
// producer calls stores_done() in every wave, then a workgroup barrier, and only then signals.
__device__ __forceinline__ float ld_agent(const float *p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ void st_agent(float *p, float v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ void stores_done() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// Values that are the same in every lane but arrive through vector loads: pin them to scalars.
__device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }
template <typename T>
__device__ __forceinline__ T *uniform_ptr(T *p) {
  const uintptr_t u = (uintptr_t)p;
  const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)u);
  const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(u >> 32));
  return (T *)(((uintptr_t)hi << 32) | lo);
}

// ---------------------------------------------------------------- numeric helpers
__device__ __forceinline__ float bf16_bits_to_float(uint32_t hi16_in_low) {
  return __uint_as_float(hi16_in_low << 16);
}

__device__ __forceinline__ bf16_t float_to_bf16_rne(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40u);  // quiet NaN
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

template <typename WT> struct Pack;   // one 16-byte load
template <> struct Pack<float> {
  static constexpr int N = 4;
  static __device__ __forceinline__ void unpack(const uint4 &u, float (&f)[4]) {
    f[0] = __uint_as_float(u.x); f[1] = __uint_as_float(u.y);
    f[2] = __uint_as_float(u.z); f[3] = __uint_as_float(u.w);
  }
  static __device__ __forceinline__ float to_float(float v) { return v; }
  static __device__ __forceinline__ float from_float(float v) { return v; }
};
template <> struct Pack<bf16_t> {
  static constexpr int N = 8;
  static __device__ __forceinline__ void unpack(const uint4 &u, float (&f)[8]) {
    f[0] = __uint_as_float(u.x << 16); f[1] = __uint_as_float(u.x & 0xffff0000u);
    f[2] = __uint_as_float(u.y << 16); f[3] = __uint_as_float(u.y & 0xffff0000u);
    f[4] = __uint_as_float(u.z << 16); f[5] = __uint_as_float(u.z & 0xffff0000u);
    f[6] = __uint_as_float(u.w << 16); f[7] = __uint_as_float(u.w & 0xffff0000u);
  }
  static __device__ __forceinline__ float to_float(bf16_t v) { return __uint_as_float((uint32_t)v << 16); }
  static __device__ __forceinline__ bf16_t from_float(float v) { return float_to_bf16_rne(v); }
};


// v of the lane that a DPP control selects inside the lane's row of 16 (a VALU move, no LDS traffic).
template <int CTRL>
__device__ __forceinline__ float dpp_row(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true));
}
// Sum over aligned groups of GS consecutive lanes (GS = 8, 16 or 32); every lane gets its group's sum.
// Within a row of 16 lanes the partners come from DPP: lanes ^1 and ^2 by quad permutation, then the
// mirrored lane of the 8-lane half and of the row (after the earlier steps every lane of a 4- or
// 8-lane block holds the block's sum, so the mirrored lane holds what lane ^4 / ^8 holds).
template <int GS>
__device__ __forceinline__ float group_sum(float v) {
  static_assert(GS == 8 || GS == 16 || GS == 32, "group sizes of the attention kernels");
  v += dpp_row<0xB1>(v);                       // quad_perm [1,0,3,2]
  v += dpp_row<0x4E>(v);                       // quad_perm [2,3,0,1]
  v += dpp_row<0x141>(v);                      // row_half_mirror
  if (GS >= 16) v += dpp_row<0x140>(v);        // row_mirror
  if (GS >= 32) v += __shfl_xor(v, 16, kWave);
  return v;
}

__device__ __forceinline__ float wave_sum(float v) {
  v = group_sum<16>(v);                        // within each row of 16 lanes, on the VALU
  v += __shfl_xor(v, 16, kWave);
  v += __shfl_xor(v, 32, kWave);
  return v;
}

// Sum over the workgroup; every thread gets the result.  red: >= kWavesPerBlock floats of LDS.
__device__ __forceinline__ float block_sum(float v, float *red) {
  v = wave_sum(v);
  __syncthreads();   // red may still be read from a previous use
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  float s = 0.f;
#pragma unroll
  for (int w = 0; w < kWavesPerBlock; ++w) s += red[w];
  return s;
}

// (value, index) ordering for argmax: larger value wins, equal values -> lower index wins.
__host__ __device__ __forceinline__ bool better(float v, int i, float bv, int bi) {
  return (v > bv) || (v == bv && i < bi);
}
// The reduction starts from (-inf, kNoIndex); a NaN never wins a comparison, so a row of NaN logits (NaN or Inf
// weights, an overflow) leaves kNoIndex standing.  The token that leaves the reduction is then token 0: an id
// inside the vocabulary, so the next step's embedding read stays inside the table.
constexpr int kNoIndex = 0x7fffffff;
__host__ __device__ __forceinline__ int argmax_token(int best_index, int vocab) {
  return (unsigned)best_index < (unsigned)vocab ? best_index : 0;
}

__device__ __forceinline__ void wave_argmax(float &v, int &i) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    float ov = __shfl_xor(v, o, kWave);
    int oi = __shfl_xor(i, o, kWave);
    if (better(ov, oi, v, i)) { v = ov; i = oi; }
  }
}

// ---------------------------------------------------------------- weight-streaming dot products
// A wave streams R rows at a time, KB column blocks per trip (R*KB independent 16-byte loads in
// flight per lane).  Lane l owns columns (blk*64 + l)*N .. +N of every row; a lane past the end of
// a ragged last block re-reads the row's last 16 bytes and its products are skipped.  The first
// trip is issued by the caller BEFORE its prologue (state is known, input vector not yet staged):
// the weights a wave reads never depend on activations, so the prologue's latency chain runs under
// the first loads.  Per row the FMA chain runs in increasing column order; the reduction order is
// fixed (no atomics), which keeps every scheduling mode bitwise identical.
// Layout of a staged input vector in LDS.  Lane l of a wave multiplies columns (blk*64 + l)*N .. +N
// (N = elements per 16-byte weight load).  Stored in plain order, a lane's N = 8 floats are 32 bytes
// and consecutive lanes sit 32 bytes apart: two-dword reads then hit 4 of the 32 banks (16-way
// conflict), which made the reads of x, not the weight stream, the limit.  So each block of 64*N
// elements is stored as N/4 planes of 64 float4: plane q holds elements 4q..4q+3 of every lane, and
// a wave reads a plane with one conflict-free 16-byte access per lane.  (N = 4: the identity.)
// The buffer is padded to whole blocks.
template <typename WT>
__host__ __device__ __forceinline__ int xs_pos(int i) {
  constexpr int N = 16 / (int)sizeof(WT);
  if (N == 4) return i;
  return (i & ~511) | (((i >> 2) & 1) << 8) | (((i >> 3) & 63) << 2) | (i & 3);
}
__host__ __device__ __forceinline__ int xs_floats(int elem_bytes, int C) {
  const int blk = 64 * (16 / elem_bytes);
  return (C + blk - 1) / blk * blk;
}

template <typename WT, int R, int KB>
struct Trip {
  uint4 u[R * KB];
};

template <typename WT>
__device__ __forceinline__ int col_blocks(int C) { return (C + kWave * Pack<WT>::N - 1) / (kWave * Pack<WT>::N); }

template <typename WT, int R, int KB>
__device__ __forceinline__ void trip_load(Trip<WT, R, KB> &t, const WT *const (&rows)[R], int cb, int nblk, int C) {
  constexpr int N = Pack<WT>::N;
  constexpr int kStride = kWave * N;
  const int lane = threadIdx.x & 63;
  const int last = C - N;
#pragma unroll
  for (int k = 0; k < KB; ++k) {
    if (cb + k < nblk) {   // wave-uniform
      const int c = min((cb + k) * kStride + lane * N, last);
#pragma unroll
      for (int r = 0; r < R; ++r) t.u[r * KB + k] = ld16_stream(rows[r] + c);
    } else {
#pragma unroll
      for (int r = 0; r < R; ++r) t.u[r * KB + k] = make_uint4(0u, 0u, 0u, 0u);
    }
  }
}

template <typename WT, int R, int KB>
__device__ __forceinline__ void trip_consume(const Trip<WT, R, KB> &t, const float *xs, int cb, int C,
                                             float (&acc)[R]) {
  constexpr int N = Pack<WT>::N;
  constexpr int kStride = kWave * N;
  const int lane = threadIdx.x & 63;
#pragma unroll
  for (int k = 0; k < KB; ++k) {
    const int c = (cb + k) * kStride + lane * N;
    if (c < C) {
      float x[N];
#pragma unroll
      for (int q = 0; q < N / 4; ++q) {
        const float4 v = *(const float4 *)(xs + (cb + k) * kStride + q * (4 * kWave) + lane * 4);
        x[4 * q] = v.x; x[4 * q + 1] = v.y; x[4 * q + 2] = v.z; x[4 * q + 3] = v.w;
      }
#pragma unroll
      for (int r = 0; r < R; ++r) {
        float w[N];
        Pack<WT>::unpack(t.u[r * KB + k], w);
#pragma unroll
        for (int e = 0; e < N; ++e) acc[r] = fmaf(w[e], x[e], acc[r]);
      }
    }
  }
}

// Sum over a workgroup of BLOCK threads; every thread gets the result.  red: BLOCK/64 floats of LDS.
template <int BLOCK>
__device__ __forceinline__ float wg_sum(float v, float *red) {
  v = wave_sum(v);
  __syncthreads();   // red may still be read from a previous use
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  float s = 0.f;
#pragma unroll
  for (int w = 0; w < BLOCK / kWave; ++w) s += red[w];
  return s;
}

// Input staging of a weight-streaming kernel, split in two so that the loads of the input vector
// can be in flight while the device state is still being read: *_issue puts the vector (and the
// norm gain) into registers, *_finish reduces and writes LDS.  A residual slot that does not depend
// on the state (the stage's working slot) is loaded before stage_in() resolves; the embedding row
// and the hExit buffers are loaded after it.
constexpr int kNormPer = 4;    // 16-byte pieces per thread: d <= 4 * kNormPer * BLOCK
constexpr int kCopyPer = 8;    // C <= 4 * kCopyPer * BLOCK

// Four consecutive elements of a storage-dtype row as floats.
__device__ __forceinline__ float4 load4_as_float(const float *p) { return *(const float4 *)p; }
__device__ __forceinline__ float4 load4_as_float(const bf16_t *p) {
  const uint2 u = *(const uint2 *)p;
  return make_float4(__uint_as_float(u.x << 16), __uint_as_float(u.x & 0xffff0000u), __uint_as_float(u.y << 16),
                     __uint_as_float(u.y & 0xffff0000u));
}

template <typename WT, int BLOCK>
struct NormStage {
  float4 xv[kNormPer], gv[kNormPer];
  // xrow (storage dtype) or xf (fp32): exactly one is non-null.  d % 4 == 0.
  __device__ __forceinline__ void issue(const float *xf, const WT *xrow, const float *gain, int d) {
#pragma unroll
    for (int e = 0; e < kNormPer; ++e) {
      const int i = 4 * (threadIdx.x + e * BLOCK);
      xv[e] = make_float4(0.f, 0.f, 0.f, 0.f); gv[e] = xv[e];
      if (i < d) {
        xv[e] = xrow ? load4_as_float(xrow + i) : load4_as_float(xf + i);
        gv[e] = load4_as_float(gain + i);
      }
    }
  }
  // RMSNorm (step a2): xs[i] = x[i] / sqrt(mean(x^2) + eps) * gain[i].  If copy_out != nullptr the
  // un-normalised x is also written there (one workgroup passes it).
  __device__ __forceinline__ void finish(int d, float eps, float *xs, float *red, float *copy_out) {
    float ss = 0.f;
#pragma unroll
    for (int e = 0; e < kNormPer; ++e) {
      const int i = 4 * (threadIdx.x + e * BLOCK);
      if (i < d) {
        if (copy_out) *(float4 *)(copy_out + i) = xv[e];
        ss = fmaf(xv[e].x, xv[e].x, ss); ss = fmaf(xv[e].y, xv[e].y, ss);
        ss = fmaf(xv[e].z, xv[e].z, ss); ss = fmaf(xv[e].w, xv[e].w, ss);
      }
    }
    ss = wg_sum<BLOCK>(ss, red);
    const float rs = 1.0f / sqrtf(ss / (float)d + eps);
#pragma unroll
    for (int e = 0; e < kNormPer; ++e) {
      const int i = 4 * (threadIdx.x + e * BLOCK);
      if (i < d)
        *(float4 *)(xs + xs_pos<WT>(i)) = make_float4(xv[e].x * rs * gv[e].x, xv[e].y * rs * gv[e].y, xv[e].z * rs * gv[e].z,
                                                      xv[e].w * rs * gv[e].w);
    }
    __syncthreads();
  }
};

template <int BLOCK, int PER = kCopyPer>
struct CopyStage {
  float4 xv[PER];
  __device__ __forceinline__ void issue(const float *vin, int C) {   // C % 4 == 0, C <= 4 * PER * BLOCK
#pragma unroll
    for (int e = 0; e < PER; ++e) {
      const int i = 4 * (threadIdx.x + e * BLOCK);
      xv[e] = i < C ? *(const float4 *)(vin + i) : make_float4(0.f, 0.f, 0.f, 0.f);
    }
  }
  template <typename WT>
  __device__ __forceinline__ void finish(int C, float *xs) {
#pragma unroll
    for (int e = 0; e < PER; ++e) {
      const int i = 4 * (threadIdx.x + e * BLOCK);
      if (i < C) *(float4 *)(xs + xs_pos<WT>(i)) = xv[e];
    }
    __syncthreads();
  }
};

// Workgroups of a weight-streaming kernel that take part (the others return at once).  In a full
// two-stage step the draft stage (E layers + exit head) runs beside the verify stage (N-E layers +
// LM head) and has a fraction of its bytes to move: with equal grids it would finish early and leave
// the verify chain alone with its launch gaps for the rest of the step.  Working with a share of its
// grid, it streams at a matching share of the bandwidth and stays beside the verify chain for the
// whole step.  A draft-only step (nothing runs beside it) uses the whole grid.  Row sums do not
// depend on which wave computes them, so results are the same bit for bit.
__device__ __forceinline__ int active_workgroups(const Common &c, int role) {
  int n = gridDim.x;
  if (role == kDraft && c.dm.draft_share < 256 && c.st->full) {
    n = (n * c.dm.draft_share + 255) >> 8;
    if (n < 1) n = 1;
  }
  return n;
}

// A residual selector whose address does not depend on the device state.
__device__ __forceinline__ bool static_slot(int sel) {
  return sel == kXDraft || sel == kXVerify || (sel >= kXStageWork0 && sel < kXStageWork0 + kMaxStages);
}

// A wave's share of a GEMV: tasks task, task + tw, ... of kTripRows rows each.  set_rows(t) points
// rows[] at task t; the first trip of `task` is already in flight in trip.  After a task's last
// trip is consumed the first trip of the wave's next task is issued before the reduction and the
// epilogue epi(task, sum_row0, sum_row1) run.
template <typename WT, typename RowsFn, typename EpiFn>
__device__ __forceinline__ void gemv_tasks(Trip<WT, kTripRows, kTripBlocks> &trip, const WT *(&rows)[kTripRows],
                                           int task, int n_tasks, int tw, int C, const float *xs,
                                           RowsFn &&set_rows, EpiFn &&epi) {
  const int nblk = col_blocks<WT>(C);
  while (task < n_tasks) {
    float acc[kTripRows] = {0.f, 0.f};
    const int next = task + tw;
    for (int cb = 0; cb < nblk; cb += kTripBlocks) {
      trip_consume<WT, kTripRows, kTripBlocks>(trip, xs, cb, C, acc);
      if (cb + kTripBlocks < nblk) {
        trip_load<WT, kTripRows, kTripBlocks>(trip, rows, cb + kTripBlocks, nblk, C);
      } else if (next < n_tasks) {
        set_rows(next);
        trip_load<WT, kTripRows, kTripBlocks>(trip, rows, 0, nblk, C);
      }
    }
    const float s0 = wave_sum(acc[0]), s1 = wave_sum(acc[1]);
    epi(task, s0, s1);
    task = next;
  }
}

// The walk of gemv_tasks with DEPTH trips in flight per wave (1 or 2), all requested before the kernel's
// prologue: start() issues them where gemv_tasks' caller issued its first trip, run() walks the tasks and
// requests trip i + DEPTH as soon as trip i's registers are free.  Per row the products are added in the
// same order whatever the depth: the sums are the same bit for bit.  epi(task, sums[R]).
// Depth 1 is gemv_tasks.  Depth 2 costs 16-18 registers (two workgroups per compute unit stay resident
// instead of three) and pays when several kernel chains run side by side: with three chains sharing the
// chip a wave waits longer for every trip, and the second trip keeps its requests queued meanwhile
// (three-stage schedule: 7B 384 -> 394, 13B 207.7 -> 211.5 tokens/s); a single chain loses 0.5-1.5 %.
template <typename WT, int R, int KB, int DEPTH>
struct Trips {
  static_assert(DEPTH == 1 || DEPTH == 2, "one or two trips in flight");
  Trip<WT, R, KB> a, b;
  int lt, lcb;                                  // the trip requested last
  template <typename RowsFn>
  __device__ __forceinline__ void next(Trip<WT, R, KB> &dst, const WT *(&rows)[R], int n_tasks, int tw, int nblk, int C,
                                       RowsFn &&set_rows) {
    lcb += KB;
    if (lcb >= nblk) { lcb = 0; lt += tw; }
    if (lt < n_tasks) {
      if (lcb == 0) set_rows(lt);
      trip_load<WT, R, KB>(dst, rows, lcb, nblk, C);
    }
  }
  template <typename RowsFn>
  __device__ __forceinline__ void start(const WT *(&rows)[R], int task, int n_tasks, int tw, int C, RowsFn &&set_rows) {
    const int nblk = col_blocks<WT>(C);
    lt = task; lcb = 0;
    if (task < n_tasks) {
      set_rows(task);
      trip_load<WT, R, KB>(a, rows, 0, nblk, C);
      if (DEPTH == 2) next(b, rows, n_tasks, tw, nblk, C, set_rows);
    }
  }
  template <typename RowsFn, typename EpiFn>
  __device__ __forceinline__ void run(const WT *(&rows)[R], int task, int n_tasks, int tw, int C, const float *xs,
                                      RowsFn &&set_rows, EpiFn &&epi) {
    const int nblk = col_blocks<WT>(C);
    int ct = task, ccb = 0;                     // the trip multiplied next
    float acc[R];
#pragma unroll
    for (int r = 0; r < R; ++r) acc[r] = 0.f;
    auto step = [&](Trip<WT, R, KB> &t) {
      trip_consume<WT, R, KB>(t, xs, ccb, C, acc);
      next(t, rows, n_tasks, tw, nblk, C, set_rows);
      ccb += KB;
      if (ccb >= nblk) {
        float s[R];
#pragma unroll
        for (int r = 0; r < R; ++r) { s[r] = wave_sum(acc[r]); acc[r] = 0.f; }
        epi(ct, s);
        ccb = 0;
        ct += tw;
      }
    };
    while (ct < n_tasks) {
      step(a);
      if (DEPTH == 2) {
        if (!(ct < n_tasks)) break;
        step(b);
      }
    }
  }
  // The same walk for ONE row per task (R = 1) whose FMA chain is handed in and out per lane instead of being
  // reduced: begin(task) gives the lane's running sum so far (0, or what an earlier column slab left), end(task,
  // sum) takes it back.  Used by the projection that walks its columns in slabs.
  template <typename RowsFn, typename BeginFn, typename EndFn>
  __device__ __forceinline__ void run_chained(const WT *(&rows)[R], int task, int n_tasks, int tw, int C, const float *xs,
                                              RowsFn &&set_rows, BeginFn &&begin, EndFn &&end) {
    static_assert(R == 1, "one row per task");
    const int nblk = col_blocks<WT>(C);
    int ct = task, ccb = 0;
    float acc[1] = {0.f};
    auto step = [&](Trip<WT, R, KB> &t) {
      if (ccb == 0) acc[0] = begin(ct);
      trip_consume<WT, R, KB>(t, xs, ccb, C, acc);
      next(t, rows, n_tasks, tw, nblk, C, set_rows);
      ccb += KB;
      if (ccb >= nblk) {
        end(ct, acc[0]);
        ccb = 0;
        ct += tw;
      }
    };
    while (ct < n_tasks) {
      step(a);
      if (DEPTH == 2) {
        if (!(ct < n_tasks)) break;
        step(b);
      }
    }
  }
};

}  // namespace ppsd
