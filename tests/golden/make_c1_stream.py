"""Writes c1_greedy_stream.txt: the oracle's greedy stream for workload C1.

Calls only the CPU oracle and the seeded input generator.  Run from the repo
root:  python tests/golden/make_c1_stream.py
"""
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import synth_inputs as S                     # noqa: E402
from oracle import decoder_fp64 as O         # noqa: E402
from oracle import ppsd_schedule as P        # noqa: E402


def main():
    w = S.WORKLOADS["C1"]
    dec = O.Decoder(w, S.make_weights(w))
    prompt = S.make_prompt(w)
    tr = O.greedy_decode(dec, prompt, w.decode_len + 1)
    ss = P.prefill(dec, prompt, w.prompt_len + w.decode_len + 2)
    toks = [ss.last_token] + P.decode(ss, w.decode_len)
    assert toks == tr.tokens
    st = ss.stats
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "c1_greedy_stream.txt")
    with open(path, "w") as f:
        f.write("# Oracle output for workload C1 (tiny fp32 decoder, seed 2509, prompt 16, 1 + 64 tokens).\n")
        f.write("# Written by tests/golden/make_c1_stream.py from oracle/ only; not a value from the paper.\n")
        f.write(f"# ppsd accepted {st.accepted} rejected {st.rejected} draft_only_steps {st.steps_draft_only}\n")
        f.write("# columns: index token top2_margin max_abs_logit\n")
        for k, (t, m, a) in enumerate(zip(tr.tokens, tr.margin, tr.absmax)):
            f.write(f"{k} {t} {m:.9e} {a:.9e}\n")
    print(path, "distinct tokens:", len(set(tr.tokens)), "accepted:", st.accepted, "rejected:", st.rejected)


if __name__ == "__main__":
    main()
