"""The shape lists and the timing protocol printed in the paper (tests/golden/paper_shapes.txt)
against what the package uses."""
import os

from paper_2601_12698_amd import binding as B
from paper_2601_12698_amd import report as R
from paper_2601_12698_amd import workloads as W

HERE = os.path.dirname(os.path.abspath(__file__))


def load_golden():
    shapes, protocol = {}, None
    for line in open(os.path.join(HERE, "golden", "paper_shapes.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        f = line.split()
        if f[0] == "PROTOCOL":
            protocol = (int(f[1]), int(f[2]))
        else:
            shapes.setdefault(f[0], []).append(tuple(int(v) for v in f[2:]))
    return shapes, protocol


def test_shape_lists_match_the_paper():
    shapes, _ = load_golden()
    assert tuple(shapes["K1"]) == W.MERGE_SHAPES
    assert shapes["K2"] == R.PAPER_MN_FP32
    assert shapes["K3"] == R.PAPER_MN_16BIT
    assert (len(shapes["K1"]), len(shapes["K2"]), len(shapes["K3"])) == (5, 8, 5)


def test_default_confirmation_protocol_is_the_papers():
    """With a zeroed budget the Top-K re-test uses the paper's warm-up and repetition counts."""
    _, protocol = load_golden()
    seen = set()

    def measure(c, warmup, reps):
        seen.add((warmup, reps))
        return 10.0 + 0.001 * c.threads_per_row
    B.addrms_tune_with_backend(64, 4096, "bf16", B.make_budget(max_candidates=8), measure)
    assert protocol == (20, 100) and protocol in seen


def test_every_paper_shape_has_a_feasible_region():
    shapes, _ = load_golden()
    for n, h, d in shapes["K1"]:
        for dt in ("bf16", "fp16"):
            assert len(B.mergestates_enumerate_feasible(n * h, d, dt)[0]) > 50
    for m, n in shapes["K2"]:
        assert len(B.addrms_enumerate_feasible(m, n, "fp32")[0]) > 50
    for m, n in shapes["K3"]:
        for dt in ("bf16", "fp16"):
            assert len(B.addrms_enumerate_feasible(m, n, dt)[0]) > 50
