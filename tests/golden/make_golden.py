"""Rewrites the stored expected values under tests/golden/ from the CPU oracle alone.

    python tests/golden/make_golden.py            # rewrite the files
    python tests/golden/make_golden.py --check    # exit 1 if a committed file differs

Every number in pick_tier_example.txt and profile_db_example.txt is computed here by calling
oracle/oracle.py (pick_tier, profile_estimate); nothing under the HIP package is imported.  The
comment lines carry the same arithmetic worked by hand, so each file checks the oracle against the
paper's rule (Section 3: inference phase, and profiler-based timing estimation) twice.
"""
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

from oracle import oracle as O  # noqa: E402


def _num(v):
    return repr(float(v))


def pick_tier_text():
    est = [2.0, 2.5, 4.0, 7.0, 13.0, 100.0, 195.0, 380.0, 760.0, 1500.0, 3000.0]
    notes = {
        100: "#  100: 1:200  4:25*2.5=62.5  16:7*4=28  32:4*7=28  64:2*13=26  512:100 ...      -> 64",
        33: "#   33: 1:66   4:9*2.5=22.5   16:3*4=12  32:2*7=14  64:13                          -> 16",
        16: "#   16: 1:32   4:4*2.5=10     16:4       32:7                                      -> 16",
        5: "#    5: 1:10   4:2*2.5=5      16:4                                                 -> 16",
        1: "#    1: 1:2    4:2.5                                                               -> 1",
        3000: "# 3000: 512:6*100=600  1024:3*195=585  2048:2*380=760  4096:760  64:47*13=611      -> 1024",
        40000: "# 40000: 16384:3*3000=9000  8192:5*1500=7500  4096:10*760=7600  2048:20*380=7600  1024:40*195=7800  -> 8192",
    }
    out = ["# Worked example of PickTier (paper Section 3, inference phase: the tier minimising",
           "# ceil(newTokens / tierSize) * estimatedSchedTime over the tier set J), computed by hand.",
           "# est_ms per tier of J = " + " ".join(str(t) for t in O.TIER_TOKENS) + ":",
           "est " + " ".join(_num(e) for e in est),
           "# tokens -> tier_tokens iterations total_ms"]
    for tokens, note in notes.items():
        tier, iters, total = O.pick_tier(est, tokens)
        out.append(note)
        out.append("case %d %d %d %s" % (tokens, O.TIER_TOKENS[tier], iters, _num(total)))
    return "\n".join(out) + "\n"


def profile_db_text():
    entries = [(1, 4, 0, 1024, 1024, 64, 0.5), (1, 4, 0, 4096, 1024, 64, 1.0), (0, 4, 0, 1024, 1024, 1, 0.01),
               (2, 4, 16, 1024, 1024, 1, 0.1), (3, 0, 0, 1048576, 1, 1, 0.02)]
    queries = [
        (["# exact match: the entry's own time"], 1000, (1, 4, 0, 1024, 1024, 64)),
        (["# neighbour: (2048, 1024, 64) is one octave from both GEMM entries: the earlier one (0.5 ms) is kept.",
          "#  its FLOPS roof = 2*1024*1024*64 / 0.5e-3 = 268435456000 flop/s.  query: flops = 2*2048*1024*64 = 268435456,",
          "#  bytes = 2048*1024*0.5625 + 2*64*(1024+2048) = 1179648 + 393216 = 1572864; intensity 170.67 flop/B;",
          "#  ridge at 1000 GB/s = 268435456000 / 1e12 = 0.268 flop/B: right of it, compute-bound: 268435456 / 268435456000 s = 1 ms"],
         1000, (1, 4, 0, 2048, 1024, 64)),
        (["#  the same query against a 1 GB/s memory roof: ridge 268.4 flop/B, memory-bound: 1572864 / 1e9 s = 1.572864 ms"],
         1, (1, 4, 0, 2048, 1024, 64)),
        (["# neighbour by distance: (8192, 1024, 64) is 1 octave from the 4096 entry, 3 from the 1024 one.",
          "#  roof = 2*4096*1024*64 / 1e-3 = 536870912000 flop/s; flops = 1073741824; at 1000 GB/s compute-bound: 2 ms"],
         1000, (1, 4, 0, 8192, 1024, 64)),
        (["# other thread count, other quantisation, or an op the database has never seen: skipped"],
         1000, (2, 4, 8, 1024, 1024, 1)),
        ([], 1000, (1, 8, 0, 1024, 1024, 64)),
        (["# copy of 4 MiB from a 1 MiB entry at 0.02 ms: same rate, 0.08 ms"], 1000, (3, 0, 0, 4194304, 1, 1)),
    ]
    out = ["# Profile database look-up (Section 3, profiler-based timing estimation), worked by hand.",
           "# entry lines:  E op quant threads n k m ms          (op 0 GEMV, 1 GEMM, 2 CPU, 3 H2D copy)",
           "# query lines:  Q bandwidth_gbps op quant threads n k m -> expected_ms match",
           "# Work of a query: flops = 2 n k m; bytes = n k (quant/8 + 1/16) + 2 m (k + n)."]
    for e in entries:
        out.append("E %d %d %d %d %d %d %s" % (e[:6] + (_num(e[6]),)))
    for notes, bw, q in queries:
        ms, match = O.profile_estimate(entries, float(bw), *q)
        out += notes
        out.append("Q %d %d %d %d %d %d %d -> %s %s" % ((bw,) + q + (_num(round(ms, 9)), match)))
    return "\n".join(out) + "\n"


FILES = {"pick_tier_example.txt": pick_tier_text, "profile_db_example.txt": profile_db_text}


def main(check):
    bad = 0
    for name, make in FILES.items():
        path, text = os.path.join(HERE, name), make()
        if check:
            same = os.path.exists(path) and open(path).read() == text
            print("%s: %s" % (name, "up to date" if same else "DIFFERS from what the oracle writes"))
            bad += 0 if same else 1
        else:
            with open(path, "w") as f:
                f.write(text)
            print("wrote", path)
    return 1 if bad else 0


if __name__ == "__main__":
    sys.exit(main("--check" in sys.argv[1:]))
