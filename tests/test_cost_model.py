"""The cost model of Sec. 3.2 (Eq. 3-6) with MI355X quantities: closed-form checks."""
import math

from paper_2509_01229_amd import cost_model as C


def test_terms_match_the_equations_by_hand():
    r = C.Rates(mem_bytes_per_s=1e12, mma_ops_per_s=1e15, valu_lane_ops_per_s=1e13)
    p = C.predict(M=16, N=1000, K=2000, group=64, rates=r, m_tile=128, alpha=2.0)
    nk = 2e6
    assert math.isclose(p["T_LD"], nk * (0.5 + 2 / 64) / 1e12)
    assert math.isclose(p["T_DQ"], 2.0 * nk / 1e13)
    assert math.isclose(p["T_MMA"], 16 * 2 * nk / 1e15)
    assert p["row_tiles"] == 1
    assert math.isclose(p["serial"], max(p["T_LD"], p["T_DQ"] + p["T_MMA"]))
    assert math.isclose(p["overlapped"], max(p["T_LD"], p["T_DQ"], p["T_MMA"]))
    # beyond one tile of rows the whole pass repeats (Eq. 6: ceil(M / M_t) in front)
    p2 = C.predict(M=300, N=1000, K=2000, group=64, rates=r, m_tile=128, alpha=2.0)
    assert p2["row_tiles"] == 3 and math.isclose(p2["T_MMA"], 128 * 2 * nk / 1e15)
    assert math.isclose(p2["serial"], 3 * max(p2["T_LD"], p2["T_DQ"] + p2["T_MMA"]))


def test_ridge_and_budgets_at_nominal_rates():
    # T_LD = T_MMA at M* = Phi_TC * bytes_per_weight / (2 * Phi_BD)
    assert math.isclose(C.ridge_batch(64), 5.033e15 * (0.5 + 2 / 64) / (2 * 8e12))
    assert 166 < C.ridge_batch(64) < 168 and 161 < C.ridge_batch(128) < 163
    # W8A8 moves twice the bytes and has no parameters: its ridge is at twice the batch of pure 4-bit
    assert math.isclose(C.ridge_batch(64, weight_bits=8), 5.033e15 / (2 * 8e12))
    # LiquidQuant's 0.94 instructions per weight fit both budgets with room to spare
    b = C.alpha_budget(M=16)
    assert C.ALPHA_LQQ < b["vs_load"] and math.isclose(b["vs_load"], (0.5 + 2 / 64) / 8e12 * 256 * 64 * 2.4e9)
    assert math.isclose(C.alpha_budget(M=4096)["vs_mma"], 128 * 2 / 5.033e15 * 256 * 64 * 2.4e9)
    # memory-bound below the ridge; above it compute-bound only if the row tile itself is
    # taller than the ridge (the intensity is bounded by M_t, Sec. 3.3): 256 rows are, 128 not
    lo, hi = C.predict(16, 8192, 8192), C.predict(4096, 8192, 8192, m_tile=256)
    assert lo["overlapped"] == lo["T_LD"] and hi["overlapped"] == hi["row_tiles"] * hi["T_MMA"]
    hi128 = C.predict(4096, 8192, 8192, m_tile=128)
    assert hi128["overlapped"] == hi128["row_tiles"] * hi128["T_LD"] > hi["overlapped"]
    # W8A8 in the memory-bound regime takes about twice as long (the paper's expectation)
    w8 = C.predict(16, 8192, 8192, weight_bits=8)
    assert 1.8 < w8["overlapped"] / lo["overlapped"] < 2.0
