"""Writes the stored expected values under tests/golden/ that are not the paper's own.
Calls only oracle/ (never the HIP path).  Run: python tests/golden/make_golden.py"""
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))
import oracle  # noqa: E402


def generator_words():
    lines = ["# seed m w salt word(hex): 32-bit words of the R generator, written by the oracle.",
             "# Both implementations (CPU oracle, HIP kernels) are compared against these."]
    for seed in (0, 1, 0x123456789ABCDEF):
        for m in (0, 1, 8191):
            for w in (0, 1, 2, 3, 4194303):
                for salt in (0, 1):
                    lines.append("%d %d %d %d %08x" % (seed, m, w, salt,
                                                       oracle.word(seed, m, w, salt)))
    open(os.path.join(HERE, "generator_words.txt"), "w").write("\n".join(lines) + "\n")


if __name__ == "__main__":
    generator_words()
