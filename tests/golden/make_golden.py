"""Writes the stored expected values under tests/golden/.

Calls only ``oracle/`` (and the seeded input generator); never the HIP path.
  closed_forms.json : values fixed by Eq.5 of arXiv 2502.05431 (Section 4.4) when
                      every key is zero -- pure arithmetic, no oracle involved.
  cfg1_oracle.json  : a sample of the oracle's output on workload 1 (T=0.8, S=0.9),
                      a regression guard for the oracle itself.
Run from the repository root:  python tests/golden/make_golden.py
"""
import json
import math
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

from oracle import ape_oracle                      # noqa: E402
from paper_2502_05431_amd import workloads as W    # noqa: E402


def main():
    # Eq.5 with all scores 0: context mass = M^S / (l_P + M^S + n_self); workload 1 has
    # l_P = 8, M = 4 x 32 = 128, n_self = row + 1, S = 0.9.
    M, lp, S = 128, 8, 0.9
    closed = {
        "zero_keys_cfg1_S0.9": {
            "cite": "Section 4.4 refined attention equation, all keys zero",
            "mass_by_row": [M ** S / (lp + M ** S + (r + 1)) for r in range(16)],
        }
    }
    closed["zero_keys_cfg1_S0.9"]["per_context_lse_row0"] = math.log(lp + 4 * 32 ** S + 1)
    with open(os.path.join(HERE, "closed_forms.json"), "w") as f:
        json.dump(closed, f, indent=1)

    spec = W.CONFIGS[1]
    r = W.make_request(spec, "cpu")
    n = W.to_numpy_f32
    out, lse, mass = ape_oracle.attention(n(r.q_self[:spec.q_len]), n(r.k_prefix), n(r.v_prefix), n(r.k_ctx), n(r.v_ctx),
                                          r.chunk_lens, n(r.k_self[:spec.q_len]), n(r.v_self[:spec.q_len]),
                                          0.8, 0.9)
    gold = {"cite": "oracle/ape_oracle.c ape_oracle_attention on workload 1, T=0.8 S=0.9, every 7th (row, head) pair",
            "out_sample": out[::7, :4].ravel().tolist(), "lse_sample": lse[::7].tolist(),
            "ctx_mass_sample": mass[::7].tolist()}
    with open(os.path.join(HERE, "cfg1_oracle.json"), "w") as f:
        json.dump(gold, f, indent=1)


if __name__ == "__main__":
    main()
