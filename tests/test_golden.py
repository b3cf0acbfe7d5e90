"""Host logic against the few values the paper prints for this path (tests/golden/paper_values.txt)."""
import os

from paper_2604_09975_amd import plan

HERE = os.path.dirname(os.path.abspath(__file__))


def rows():
    out = []
    for line in open(os.path.join(HERE, "golden", "paper_values.txt")):
        if line.startswith("#") or not line.strip():
            continue
        key, args, value, cite = [p.strip() for p in line.split("|")]
        out.append((key, dict((k, int(v)) for k, v in (a.split("=") for a in args.split())), int(value), cite))
    return out


def test_paper_values():
    seen = set()
    for key, a, value, cite in rows():
        assert cite, "every golden value carries its citation"
        if key == "ct_bytes":
            got = plan.ciphertext_bytes(a["N"], a["L"])
        elif key == "blocks":
            got = plan.blocks(a["d"], a["C"])
        elif key == "segments":
            got = plan.segments(a["n"], a["m"])
        elif key == "pairs":
            got = plan.complex_pairs(a["G"])
        else:
            raise AssertionError(key)
        assert got == value, (key, a, got, value, cite)
        seen.add(key)
    assert seen == {"ct_bytes", "blocks", "segments", "pairs"}


def test_layout_sizes_match_the_library_s_buffers():
    # a ciphertext buffer of the library is [2][level][N] 8-byte words: the paper's ct_bytes
    N, level = 1 << 16, 24
    assert 2 * level * N * 8 == plan.ciphertext_bytes(N, level)
