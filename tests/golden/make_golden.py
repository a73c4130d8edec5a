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


def gaussian_table():
    """The 256 table values of the Gaussian family as bfloat16 bit patterns (hex), entry i on line i."""
    import numpy as np
    T = oracle.gauss_table().astype(np.float32)
    bits = T.view(np.uint32)
    assert np.all((bits & 0xFFFF) == 0), "table entries are bfloat16 values"
    lines = ["# bfloat16 bit patterns of T[i] = bf16_rne(Phi^-1((i + 1/2) / 256)), i = 0..255, written by the oracle.",
             "# Both implementations (CPU oracle, HIP library) are compared against these."]
    lines += ["%04x" % (int(b) >> 16) for b in bits]
    open(os.path.join(HERE, "gaussian_table_bf16.txt"), "w").write("\n".join(lines) + "\n")


if __name__ == "__main__":
    generator_words()
    gaussian_table()
