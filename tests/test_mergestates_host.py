"""merge_attn_states through the same deriver and search (host logic, no GPU)."""
import math

from paper_2601_12698_amd import binding as B


def test_bytes_and_dtypes():
    assert B.mergestates_algorithmic_bytes(512 * 32, 256, "bf16") == 512 * 32 * (3 * 256 * 2 + 12)
    assert B.load().mergestates_algorithmic_bytes(16, 128, B.FP32) == B.ERR_UNSUPPORTED_DTYPE
    assert B.load().mergestates_algorithmic_bytes(16, 128, B.FP16_RES32) == B.ERR_UNSUPPORTED_DTYPE


def test_short_rows_pack_into_waves():
    for d in (128, 256, 64, 96):
        c = B.mergestates_default_cfg(d, "bf16")
        assert c.reduce == 0 and c.threads_per_row * c.rows_per_wg % 64 == 0
        assert B.mergestates_cfg_feasible(c, 16384, d, "bf16")[0] == 0
    cfgs, grid = B.mergestates_enumerate_feasible(512 * 32, 256, "bf16")
    assert len(cfgs) > 100 and all(c.reduce == 0 for c in cfgs)
    # d = 256 at vec 8 is one chunk over 32 lanes: two rows share a wave
    assert any(c.vec == 8 and c.threads_per_row == 32 and c.rows_per_wg >= 2 for c in cfgs)
    st, why, _ = B.mergestates_cfg_feasible(B.make_cfg(8, 32, 2, reduce=1), 1000, 256, "fp16")
    assert st == B.ERR_INFEASIBLE_CFG and "no reduction" in why
    st, why, _ = B.mergestates_cfg_feasible(B.make_cfg(8, 8, 8), 1000, 512, "fp16")      # 8 chunks: beyond this operator's instances
    assert st == B.ERR_INFEASIBLE_CFG and "no compiled instance" in why


def test_search_and_table_for_this_operator():
    B.addrms_table_clear()

    def measure(c, w, r):
        return 6.0 * (1 + 0.2 * abs(math.log2(c.threads_per_row * c.rows_per_wg / 256))) * (1 + 0.1 * abs(math.log2(c.vec / 8)))
    g, rep = B.mergestates_tune_with_backend(16384, 256, "bf16", B.make_budget(), measure, lambda c: True)
    assert B.mergestates_cfg_feasible(g, 16384, 256, "bf16")[0] == 0
    assert g.vec == 8 and g.threads_per_row * g.rows_per_wg == 256
    assert B.mergestates_table_lookup(16384, 256, "bf16") is None       # the backend variant does not touch the table
