"""CPU oracle for the PPSD decode path.  TEST INFRASTRUCTURE ONLY.

Plain, slow, fp64 PyTorch-CPU code written from the paper's definitions; it
shares no code with the HIP library and never imports it.  Only tests, the
smoke check and the benchmark's cpu_baseline leg may import this package; the
product path must never route through it.

Modules
  decoder_fp64   Llama-style decoder (RMSNorm, RoPE, MHA/GQA, SwiGLU) and
                 vanilla greedy autoregressive decoding: the result that
                 lossless self-speculative decoding must reproduce (Sec. 5.1,
                 "Evaluation Metrics": output aligned with auto-regressive
                 decoding); the early-exit norm head and the transformer-layer
                 exit head (Sec. 3.1, Sec. 5.4 "Impact of exit head").
  ppsd_schedule  Two-stage verify-while-draft schedule and the full pipeline
                 schedule with S stages, tick by tick (Sec. 4.1-4.2, Alg. 1:
                 compare check token with own draft, roll the index back).
  eesd_schedule  Draft-then-verify rounds of early-exit speculative decoding
                 with gamma drafts per round (Sec. 3.1, Eq. 4-5).
  stochastic     Sampled drafts and stochastic verification (Sec. 3.1,
                 Eq. 1-2) for every schedule, with a counter-based uniform
                 generator of its own.
  speedup_model  Closed forms of Eq. (3)-(8) and a tick-count model of Eq. (7).

Pins: every function is pinned by tests/test_oracle_*.py (closed forms,
invariants, brute force, library routines, the paper's worked 1.31x).  Token
values at the 7B/13B/8B shapes have no published counterpart: for those the
oracle is pinned structurally on small shapes and runs the same code at the
large ones ("parity unpinned" by the paper for the values themselves).
"""
