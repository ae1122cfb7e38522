"""Writes tests/golden/tiny_m2_n16_k16_g8.txt: a hand-checkable instance (m = 2, n = k = 16,
group_size = 8) whose digits follow closed-form patterns.  It calls neither the oracle nor the
HIP library: the expected values of the test that reads the file are expanded there, in exact
rationals, from these digits.

    python tests/golden/make_tiny_fixture.py            # rewrite the file
    python tests/golden/make_tiny_fixture.py --print    # print it instead
"""
import pathlib
import sys

OUT = pathlib.Path(__file__).resolve().parent / "tiny_m2_n16_k16_g8.txt"


def fixture_text() -> str:
    m, n, k, g = 2, 16, 16, 8
    q = [[(3 * kk + 5 * j + kk * j) % 16 for j in range(n)] for kk in range(k)]
    z = [[(7 * gi + 3 * j + 1) % 16 for j in range(n)] for gi in range(k // g)]
    se = [[-(1 + (j + gi) % 4) for j in range(n)] for gi in range(k // g)]  # scale = 2**se
    A = [[(i + 1) * ((kk * 7 + i) % 5 - 2) for kk in range(k)] for i in range(m)]
    H = "0123456789ABCDEF"
    out = [
        "# Tiny hand-checkable W4A16 instance: m=2, n=k=16, group_size=8.",
        "# Not from the paper (it prints no worked example); digits follow simple closed-form patterns",
        "# so a reader can re-derive any entry.  The test expands every dot product in exact rationals.",
        "# Layout being pinned (paper Section 2, packed int32 weights; field order is this build's reading):",
        "#   a packed word is written as 8 hex digits, most significant first;",
        "#   the RIGHTMOST digit is field 0, the LEFTMOST is field 7.",
        "#   qweight word (r, j): field i is q[8r+i][j].   qzeros word (gi, c): field i is z[gi][8c+i].",
        "[q] k rows of n hex digits: q[kk][j]",
    ]
    out += ["".join(H[v] for v in q[kk]) for kk in range(k)]
    out.append("[z] k/g rows of n hex digits: z[gi][j]")
    out += ["".join(H[v] for v in z[gi]) for gi in range(k // g)]
    out.append("[scale_exponent] k/g rows of n integers e: s[gi][j] = 2**e")
    out += [" ".join(str(v) for v in se[gi]) for gi in range(k // g)]
    out.append("[A] m rows of k integers")
    out += [" ".join(str(v) for v in A[i]) for i in range(m)]
    out.append("[qweight] k/8 rows of n words")
    out += [" ".join("".join(H[q[8 * r + i][j]] for i in reversed(range(8))) for j in range(n)) for r in range(k // 8)]
    out.append("[qzeros] k/g rows of n/8 words")
    out += [" ".join("".join(H[z[gi][8 * c + i]] for i in reversed(range(8))) for c in range(n // 8))
            for gi in range(k // g)]
    return "\n".join(out) + "\n"


if __name__ == "__main__":
    if "--print" in sys.argv[1:]:
        sys.stdout.write(fixture_text())
    else:
        OUT.write_text(fixture_text())
        print(OUT)
