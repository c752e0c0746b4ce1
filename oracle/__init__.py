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
                 decoding).
  ppsd_schedule  Two-stage verify-while-draft schedule (Sec. 4.1-4.2, Alg. 1:
                 compare check token with own draft, roll the index back).
  speedup_model  Closed forms of Eq. (3)-(8) and a tick-count model of Eq. (7).

Pins: every function is pinned by tests/test_oracle_*.py (closed forms,
invariants, brute force, library routines, the paper's worked 1.31x).  Token
values at the 7B/13B/8B shapes have no published counterpart: for those the
oracle is pinned structurally on small shapes and runs the same code at the
large ones ("parity unpinned" by the paper for the values themselves).
"""
