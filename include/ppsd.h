/*
 * ppsd.h -- C ABI of the MI355X (gfx950) library for pipeline-parallel early-exit
 * self-speculative decoding, batch 1, one GPU.
 *
 * The method (paper Sec. 3.1, 4.1, 4.2 and Alg. 1): the first E layers of a
 * decoder-only transformer plus an early-exit head draft token t+1 while layers
 * E+1..N plus the LM head verify token t, reusing the draft pass's hidden state
 * and KV cache.  The verifier's token is compared with the draft for the same
 * position; on a mismatch the draft and everything computed from it (its KV rows,
 * its hidden state, the next draft) are dropped and drafting restarts from the
 * verifier's token.  With greedy (argmax) heads the committed stream equals vanilla
 * greedy autoregressive decoding of the full model (Sec. 5.1, "Evaluation Metrics").
 *
 * Conventions
 *   - Every function returns 0 on success or a negative PPSD_E* code; it never
 *     throws.  ppsd_last_error() returns a thread-local message for the last
 *     failure on the calling thread.
 *   - Pointers marked DEVICE are HIP device pointers on the current device;
 *     pointers marked HOST are ordinary host pointers.  The caller owns all of
 *     them.  Device memory handed over in ppsd_buffers is BORROWED: it must stay
 *     alive and unmodified (weights) / untouched (workspace) until ppsd_free().
 *   - The library allocates no device memory.  It owns the host-side context, a
 *     few HIP events, captured graphs and one small pinned host block.
 *   - Calls on one context must not overlap.  The library synchronises the two
 *     streams it was given before returning from prefill/decode.
 *   - Matrices are row-major [out_features, in_features] in the storage dtype;
 *     norm gains are fp32.  Residual stream, accumulators, softmax and logits
 *     are fp32.
 */
#ifndef PPSD_H
#define PPSD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PPSD_OK         0
#define PPSD_EARG      (-1)  /* bad argument or unsupported configuration */
#define PPSD_ESTATE    (-2)  /* call out of order (e.g. decode before prefill) */
#define PPSD_ECAPACITY (-3)  /* sequence would exceed max_seq, or workspace too small */
#define PPSD_EHIP      (-4)  /* a HIP call failed; message holds hipGetErrorString */

#define PPSD_FP32 0
#define PPSD_BF16 1

/* Scheduling of one decode step (Sec. 4.1-4.2).  All modes run the same kernels. */
#define PPSD_MODE_VANILLA    0  /* autoregressive: all N layers + LM head per token, no draft */
#define PPSD_MODE_SERIAL     1  /* draft stage then verify stage on one stream */
#define PPSD_MODE_OVERLAP    2  /* draft stage and verify stage on two streams (verify-while-draft) */
#define PPSD_MODE_PIPELINE   3  /* the full schedule of Sec. 4.1-4.2 / Alg. 1: S = ceil(N/E) stages of E layers
                                   (the last takes what remains), stage 0 + exit head drafting one token per
                                   tick from its own previous draft, every later stage carrying the token it
                                   received one tick earlier, the last stage + LM head yielding the verified
                                   token.  A mismatch with the draft used at that position drops all S-1
                                   tokens in flight and restarts stage 0 from the verified token, so an
                                   accepted token costs one tick and a rejected one S ticks (Eq. 7).  On one
                                   GPU the S stages of a tick share the chip: stage k runs on stream
                                   k mod pipeline_streams.  Per-operation engine only, S <= 16, no
                                   time_kernels.  With S = 2 it commits what PPSD_MODE_OVERLAP commits. */

/* Execution engines.  Both run every step of the path in this library's HIP kernels and give
 * the same tokens; logits agree to fp32 rounding (the RMSNorm sums are grouped differently). */
#define PPSD_ENGINE_STREAMS    0  /* one kernel per operation; the stages on the two caller streams,
                                     one captured HIP graph per step if use_graph */
#define PPSD_ENGINE_PERSISTENT 1  /* one cooperative persistent kernel per prefill/decode call: grid
                                     barriers between operations, the two stages zipped phase by phase
                                     (PPSD_MODE_OVERLAP) or back to back (PPSD_MODE_SERIAL), weight
                                     loads software-pipelined across barriers.  Uses stream_draft only. */

#define PPSD_MODE_EESD       4  /* draft-then-verify rounds of early-exit speculative decoding (Sec. 3.1, Eq. 4-5),
                                   the method the pipeline is measured against: eesd_gamma draft steps (layers
                                   1..E + exit head, one token each), then ONE pass of layers E+1..N + LM head
                                   over the gamma + 1 drafted positions, every weight streamed once for all of
                                   them; the accepted prefix plus the full model's next token are committed.
                                   One stream (stream_draft).  Per-operation engine only, no time_kernels. */

typedef struct ppsd_ctx ppsd_ctx;

typedef struct {
  int32_t n_layers;        /* N (paper) */
  int32_t exit_layer;      /* E: the draft model is layers 1..E; 1 <= E < N */
  int32_t d_model;
  int32_t n_heads;         /* query heads */
  int32_t n_kv_heads;      /* n_heads / n_kv_heads in {1,2,4} */
  int32_t head_dim;        /* 64 or 128 */
  int32_t d_ffn;
  int32_t vocab;
  int32_t dtype;           /* PPSD_FP32 / PPSD_BF16: storage of weights and KV cache */
  int32_t max_seq;         /* capacity in positions (prompt + generated + speculative: 1, or S-1 in
                              PPSD_MODE_PIPELINE) */
  int32_t kv_page_tokens;  /* positions per KV page: 8, 16, 32 or 64 */
  int32_t mode;            /* PPSD_MODE_* */
  float   rope_base;       /* rotary base; pair (i, i+hd/2) turns by pos * base^(-2i/hd) */
  float   rms_eps;
  int32_t debug_logits;    /* >0: keep the LM-head logits behind the first debug_logits committed
                              tokens (token #0 = the one prefill returns) for ppsd_read_logits */
  int32_t use_graph;       /* 1: replay one captured HIP graph per step; 0: launch kernels directly */
  int32_t time_kernels;    /* 1: profiling mode -- direct launches on one stream with a HIP event
                              between consecutive kernels, totals via ppsd_kernel_times (slow) */
  int32_t engine;          /* PPSD_ENGINE_*: how a step is executed on the GPU */
  int32_t prefill_loop;    /* 0: prefill on the matrix cores (MFMA GEMMs over chunks of the prompt, see prefill_chunk) when the
                              configuration allows it (bf16, head_dim 128, d_model % 128 == 0,
                              d_ffn % 64 == 0), else the loop below; 1: always run the prompt through the
                              decode kernels one position at a time */
  int32_t pipeline_streams;/* PPSD_MODE_PIPELINE: streams the stages of a tick are spread over; 0 = default
                              (min(S, 4)), else 2..4.  Streams beyond the caller's two are created (default
                              priority) and destroyed by the library */
  int32_t tune_wgs_per_cu; /* launch tuning: workgroups per compute unit of the weight-streaming kernels,
                              1..4; 0 = the library's defaults (3; 2 for gate/up) */
  int32_t tune_attn_split; /* launch tuning: positions of capacity (max_seq) per attention split, >= 64; the
                              number of splits is capped at 64.  0 = the library's default (one split up to
                              512 positions; beyond that one per 512 or, if that is more, one per compute unit
                              and KV head, with at least 128 positions of capacity each) */
  int32_t eesd_gamma;      /* PPSD_MODE_EESD: drafts per round, 1..4; 0 = default (3).  (gamma + 1) * d_model
                              floats must fit the LDS of a compute unit (150 KiB) */
  int32_t exit_block;      /* 1: the early-exit head is one more transformer layer of the model's own structure
                              followed by the norm head (the head of the paper's main results, Sec. 5.4 "Impact of
                              exit head").  Its tensors are entry n_layers of the per-layer arrays, it keeps its
                              own KV rows (rolled back with those of layers 1..E), and its output feeds the exit
                              head only.  Per-operation engine only, no time_kernels */
  float   temperature;     /* 0: greedy heads (argmax), the default.  > 0 (>= 1e-4): stochastic verification
                              (Sec. 3.1, Eq. 1-2) in PPSD_MODE_SERIAL / OVERLAP / PIPELINE / EESD -- the draft is sampled
                              from softmax(exit logits / temperature) = p, accepted with probability
                              min(1, q(d) / p(d)) against q = softmax(LM logits / temperature), and a rejected
                              draft is replaced by a token from normalise(max(0, q - p)), so every committed token
                              is q-distributed -- and plain sampling from q in PPSD_MODE_VANILLA, for token #0 and
                              for the token behind a fully accepted draft-then-verify round.
                              Sampling is by inverse CDF in index order.  Per-operation engine only */
  uint32_t sample_seed;    /* the uniform for (position, purpose) is the top 24 bits of splitmix64's output
                              function applied to seed ^ position * 0xD1342543DE82EF95 ^ purpose *
                              0xA0761D6478BD642F (64-bit wrapping), purpose = 0 draft, 1 acceptance,
                              2 replacement, 3 plain sampling: a pure function of the three, whatever the schedule */
  int32_t prefill_chunk;   /* positions the matrix-core prefill takes through the layers at a time: 0 = default
                              (the whole prompt capacity max_seq, 4096 at most), else a multiple of 128 in
                              128..4096.  Sizes the chunk buffers inside the workspace */
  int32_t tune_prefill_tile; /* launch tuning of the matrix-core prefill GEMMs: 0 = choose per projection (256 x 256
                              output tiles when they still fill the chip, else 128 x 128 with K split over
                              several workgroups), 1 = always 128 x 128, 2 = always 256 x 256 */
  int32_t tune_draft_share;/* launch tuning of PPSD_MODE_OVERLAP: percent of their workgroups the draft stage's
                              weight-streaming kernels work with while the verify stage runs beside them (the
                              others return at once), 1..100; 0 = the library's default.  The draft stage has
                              E layers + a head to stream against N-E layers + a head: with a matching share
                              of the bandwidth it stays beside the verify chain for the whole step instead of
                              finishing early.  Draft-only steps use every workgroup.  Results do not depend
                              on it */
  int32_t pipeline_stage_layers; /* PPSD_MODE_PIPELINE: layers per stage behind the draft stage; 0 = exit_layer, the paper's
                              balanced partition into ceil(N/E) stages (one GPU each, Sec. 4.1).  On one GPU the
                              stages share the memory system and need not be equal: fewer, longer stages behind the
                              draft stage keep fewer speculative tokens in flight, so a rejection drops less work
                              (S - 1 tokens, S = 1 + ceil((N - E) / pipeline_stage_layers)), at the price of fewer
                              kernel chains running side by side.  N - E gives the two-stage schedule */
} ppsd_config;

/* DEVICE pointers, BORROWED.  Per-layer entries are HOST arrays of n_layers DEVICE pointers
 * (n_layers + 1 with exit_block: the early-exit block last). */
typedef struct {
  const void *embed;        /* [vocab, d_model] storage dtype */
  const void *final_norm;   /* [d_model] fp32 */
  const void *lm_head;      /* [vocab, d_model] */
  const void *exit_norm;    /* [d_model] fp32: gain of the early-exit norm head (Sec. 3.1) */
  const void *exit_head;    /* [vocab, d_model] */
  const void *const *attn_norm;  /* [d_model] fp32 each */
  const void *const *wqkv;       /* [(n_heads + 2 n_kv_heads) * head_dim, d_model]: q heads, k heads, v heads */
  const void *const *wo;         /* [d_model, n_heads * head_dim] */
  const void *const *mlp_norm;   /* [d_model] fp32 each */
  const void *const *wgu;        /* [2 d_ffn, d_model]: gate rows then up rows */
  const void *const *wdown;      /* [d_model, d_ffn] */
  void  *workspace;              /* >= ppsd_workspace_bytes(cfg) bytes, 256-byte aligned: KV pages,
                                    activations, device-side decode state.  Contents are the library's. */
  size_t workspace_bytes;
  void  *stream_draft;           /* hipStream_t (not the legacy default stream) */
  void  *stream_verify;          /* hipStream_t, distinct from stream_draft, same (default) priority */
  const int32_t *kv_page_table;  /* HOST, optional: permutation of 0..n_pages-1 mapping logical KV page
                                    -> physical page; NULL = identity.  n_pages = ceil(max_seq / kv_page_tokens) */
} ppsd_buffers;

/* Counters since the last ppsd_prefill (paper metrics: AR = accepted / drafts_compared, Sec. 5.1). */
typedef struct {
  int64_t committed;         /* tokens returned by ppsd_decode */
  int64_t drafts_compared;   /* drafts that met their verifier token */
  int64_t accepted;
  int64_t rejected;
  int64_t steps_overlapped;  /* steps that ran both stages */
  int64_t steps_draft_only;  /* pipeline-refill steps: draft stage only, nothing committed */
  int64_t kv_rollbacks;      /* rejected drafts whose KV rows (layers 1..E) were dropped */
  int64_t steps_launched;    /* steps the host enqueued, including ones that found nothing to do */
  double  device_ms;         /* HIP-event time spent inside ppsd_decode */
  /* PPSD_MODE_PIPELINE only (zero otherwise); there steps_overlapped / steps_draft_only count the ticks
   * in which several stages / only stage 0 ran, and kv_rollbacks the rejections. */
  int64_t pipeline_ticks;    /* ticks that did work; Eq. (7): committed + (S-1) * rejected, up to fill/drain */
  int64_t stage_runs;        /* stage executions summed over ticks */
  int64_t flushed_tokens;    /* speculative tokens in flight dropped by rejections (S-1 per rejection) */
  /* PPSD_MODE_EESD only: rounds run; there drafts_compared counts drafts up to and including a round's first
   * mismatch, accepted the accepted ones, rejected = kv_rollbacks the rounds that ended at a mismatch. */
  int64_t eesd_rounds;
} ppsd_stats_t;

#define PPSD_N_KERNEL_KINDS 7   /* qkv, attention, o_proj, gate_up, down, head, commit */
typedef struct {
  double  total_us[PPSD_N_KERNEL_KINDS];  /* sum of event-to-event intervals around ACTIVE launches */
  int64_t launches[PPSD_N_KERNEL_KINDS];
  double  event_overhead_us;              /* what one event adds to such an interval, measured on the same stream
                                             at the first profiled step: empty kernels with an event after each
                                             against empty kernels back to back.  Included in total_us */
} ppsd_kernel_times_t;

/* Bytes of workspace a context with this configuration needs.  0 if cfg is invalid. */
size_t ppsd_workspace_bytes(const ppsd_config *cfg);

/* The stage layout of Sec. 4.1 on one GPU: the model's N layers with the early-exit head behind layer E
 * (the draft model = layers 1..E + that head, Sec. 3.1) and the LM head behind layer N, all stages sharing
 * one KV cache (the verifier reuses the draft pass's rows, Sec. 3.1).
 * Validates cfg, records the borrowed pointers, builds the rotary table (computed in double on
 * the host) and the KV page table, zeroes the device state.  *out receives the context.
 * PPSD_EARG for a null / misaligned pointer or an unsupported configuration, PPSD_ECAPACITY if the workspace is
 * smaller than ppsd_workspace_bytes(cfg), PPSD_EHIP if a HIP call fails; on any error *out is NULL. */
int ppsd_load_weights(const ppsd_config *cfg, const ppsd_buffers *bufs, ppsd_ctx **out);

/* The pipeline's warm-up (Sec. 4.1: after it all stages can work in parallel; Alg. 1 starts from the prompt
 * x_1..x_n): resets the sequence, runs the full model over prompt (HOST, n_prompt >= 1 ids in [0, vocab)),
 * fills the KV cache of all layers for positions 0..n_prompt-1 and writes generated token #0 (the
 * full model's greedy token after the prompt) to *first_token (HOST).  The pipeline is left empty:
 * the first decode step is a draft-only step.  PPSD_ECAPACITY if n_prompt + 2 > max_seq. */
int ppsd_prefill(ppsd_ctx *ctx, const int32_t *prompt, int32_t n_prompt, int32_t *first_token);

/* Commits exactly n_tokens further tokens into out_tokens (HOST) and sets *n_written = n_tokens.
 * One step drafts with layers 1..E + exit head and verifies with layers E+1..N + LM head
 * (Sec. 4.2); accept/reject and KV rollback happen on the device (Alg. 1).  Resumable: a second
 * call continues the same sequence, keeping the drafts in flight.  PPSD_ESTATE before prefill;
 * PPSD_ECAPACITY if the sequence plus the speculative positions (one; S-1 in PPSD_MODE_PIPELINE;
 * eesd_gamma in PPSD_MODE_EESD) would pass max_seq. */
int ppsd_decode(ppsd_ctx *ctx, int32_t n_tokens, int32_t *out_tokens, int32_t *n_written);

/* For callers that cannot allocate device memory while they decode (tight serving loops, harnesses that
 * forbid hipMalloc, code that must not grow the process's device footprint): ppsd_decode with the per-step
 * scratch of its kernels -- the vectors between the kernels of a layer, the attention split partials and
 * their arrival counters, the heads' argmax candidates, the batched pass's vectors -- in a static device
 * array of PPSD_STATIC_SCRATCH_BYTES inside the library instead of the caller's workspace (KV cache, decode
 * state, hidden states and weights stay where ppsd_load_weights put them).  The call itself allocates
 * nothing on host or device: kernels are launched directly (no graph), the tokens come back through the
 * context's pinned block.  Same arguments, results and errors as ppsd_decode, and calls of the two may
 * alternate on one context; in addition PPSD_ECAPACITY if the configuration's scratch exceeds the static
 * region, PPSD_EARG with the persistent engine or time_kernels, PPSD_ESTATE if the current device is not
 * the context's.  Every context on a device shares that device's array (each device has its own copy, held
 * until the process ends): calls that overlap in time on one device race; run them one after the other. */
#define PPSD_STATIC_SCRATCH_BYTES (16u << 20)
int ppsd_decode_static_scratch(ppsd_ctx *ctx, int32_t n_tokens, int32_t *out_tokens, int32_t *n_written);

/* Copies the counters (HOST out). */
int ppsd_stats(const ppsd_ctx *ctx, ppsd_stats_t *out);

/* Debug/parity: logits behind committed tokens first..first+count-1 (token #0 = prefill's) into
 * out (HOST, count * vocab floats).  Needs debug_logits >= first + count. */
int ppsd_read_logits(ppsd_ctx *ctx, int32_t first, int32_t count, float *out);

/* Debug/parity: for committed tokens first..first+count-1, the draft that was compared with it,
 * or -1 if the token was committed without a draft (token #0, vanilla mode). HOST out. */
int ppsd_read_drafts(ppsd_ctx *ctx, int32_t first, int32_t count, int32_t *out);

/* What the context launches, as decided at ppsd_load_weights from the configuration and the device
 * (parity tests and benchmark reports state the launch configuration they ran in). */
typedef struct {
  int32_t compute_units;        /* of the device */
  int32_t attn_splits;          /* splits along the sequence of the decode attention (grid = n_kv_heads x splits) */
  int32_t prefill_matrix_core;  /* 1: ppsd_prefill runs the MFMA path, 0: the looped decode kernels */
  int32_t prefill_chunk;        /* positions per chunk of the MFMA prefill (0 when it is not used) */
  int32_t grid_qkv, grid_proj, grid_gate_up, grid_head;   /* workgroups of the weight-streaming kernels */
  int32_t draft_share_of_256;   /* PPSD_MODE_OVERLAP: share of its workgroups the draft stage works with beside the verify stage */
  int32_t streams;              /* streams a step is spread over */
  int32_t pipeline_stages;      /* ceil(n_layers / exit_layer) */
  int32_t eesd_gamma;           /* drafts per round in PPSD_MODE_EESD, else 0 */
} ppsd_launch_info_t;
int ppsd_launch_info(const ppsd_ctx *ctx, ppsd_launch_info_t *out);

/* Profiling mode only (time_kernels = 1): accumulated per-kind kernel durations. */
int ppsd_kernel_times(const ppsd_ctx *ctx, ppsd_kernel_times_t *out);

/* Measurement support, persistent engine: ask the next ppsd_decode calls to record, for decode step
 * `step` of each call (step < 0 switches it off), the timeline of workgroup `workgroup`: per phase
 * four 100 MHz timestamps (barrier passed, inputs staged, own weight tasks done, arrived at the next
 * barrier).  ppsd_trace_read copies 4 * n_phases values (HOST out); phases a step skipped hold stale
 * values. */
int ppsd_trace_request(ppsd_ctx *ctx, int32_t step, int32_t workgroup);
int ppsd_trace_read(ppsd_ctx *ctx, int32_t n_phases, uint64_t *out);

/* Measurement support: times `iters` launches of a pure streaming-read kernel over a DEVICE
 * buffer of `bytes` bytes on `stream` (hipStream_t) and writes the average ms per launch.
 * Gives the HBM read rate a kernel on this chip can actually reach. */
int ppsd_hbm_read_probe(const void *buf, size_t bytes, void *stream, int32_t iters, float *avg_ms);

void ppsd_free(ppsd_ctx *ctx);
const char *ppsd_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* PPSD_H */
