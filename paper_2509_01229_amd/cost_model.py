"""The paper's GEMM cost model (Sec. 3.2, Eq. 3-6) with MI355X quantities.

    T = ceil(M / M_t) * max( T_LD , T_DQ + T_MMA )                                   (Eq. 6)
    T_LD  = N K * bytes_per_weight / Phi_BD        weights streamed once per row of tiles
    T_DQ  = alpha * N K / Phi_VALU                 alpha = dequantisation instructions per weight
    T_MMA = min(M_t, M) * 2 N K / Phi_TC           one multiply-accumulate = 2 operations

Eq. 6 adds T_DQ and T_MMA because in the pipelines the paper analyses the two run one after
the other inside a compute stage; a pipeline that overlaps them (the paper's implicit
fine-grained pipeline, Sec. 5.1; here: two waves per SIMD) is bounded by the maximum of the
three terms instead.  Both forms are returned.  Pure arithmetic on Python numbers: no GPU,
no numpy; bench.py feeds it the rates it measures on the box.
"""
from __future__ import annotations

import math
from dataclasses import dataclass

# MI355X nominal figures
NOMINAL_HBM_BYTES_PER_S = 8.0e12
NOMINAL_INT8_OPS_PER_S = 5.033e15       # 256 CU x 4 SIMD x 2048 ops/clk x 2.4 GHz
NOMINAL_VALU_LANE_OPS_PER_S = 256 * 64 * 2.4e9  # 256 CU x 64 lanes/clk x 2.4 GHz (one instruction per lane)

# LiquidQuant dequantisation on gfx950: and, shift+and, 2 x pk_mad, 2 x xor per 8 codes
# (Sec. 5.3) plus 2 v_perm per 32 codes for the parameter broadcast.
ALPHA_LQQ = 7.0 / 8.0 + 2.0 / 32.0


@dataclass(frozen=True)
class Rates:
    mem_bytes_per_s: float = NOMINAL_HBM_BYTES_PER_S
    mma_ops_per_s: float = NOMINAL_INT8_OPS_PER_S
    valu_lane_ops_per_s: float = NOMINAL_VALU_LANE_OPS_PER_S


def bytes_per_weight(weight_bits: int = 4, group: int = 64) -> float:
    """Packed code plus its share of the (s_u8, a) byte pair of its group (none for 8 bits)."""
    return weight_bits / 8.0 + (2.0 / group if weight_bits == 4 else 0.0)


def terms(M, N, K, group=64, rates: Rates = Rates(), m_tile=128, weight_bits=4, alpha=ALPHA_LQQ):
    """(T_LD, T_DQ, T_MMA, row_tiles) in seconds for one row of tiles (Eq. 3, Eq. 4)."""
    nk = float(N) * K
    t_ld = nk * bytes_per_weight(weight_bits, group) / rates.mem_bytes_per_s
    t_dq = (alpha if weight_bits == 4 else 0.0) * nk / rates.valu_lane_ops_per_s
    t_mma = min(m_tile, M) * 2.0 * nk / rates.mma_ops_per_s
    return t_ld, t_dq, t_mma, math.ceil(M / m_tile)


def predict(M, N, K, group=64, rates: Rates = Rates(), m_tile=128, weight_bits=4, alpha=ALPHA_LQQ):
    """Predicted seconds: {'serial': Eq. 6 as printed, 'overlapped': max of the three terms}."""
    t_ld, t_dq, t_mma, rows = terms(M, N, K, group, rates, m_tile, weight_bits, alpha)
    return {
        "serial": rows * max(t_ld, t_dq + t_mma),
        "overlapped": rows * max(t_ld, t_dq, t_mma),
        "T_LD": t_ld, "T_DQ": t_dq, "T_MMA": t_mma, "row_tiles": rows,
    }


def ridge_batch(group=64, rates: Rates = Rates(), weight_bits=4) -> float:
    """Batch size at which T_LD = T_MMA (memory-bound below, compute-bound above; the
    counterpart of the paper's transition points of Sec. 3.3)."""
    return rates.mma_ops_per_s * bytes_per_weight(weight_bits, group) / (2.0 * rates.mem_bytes_per_s)


def alpha_budget(M, group=64, rates: Rates = Rates(), m_tile=128):
    """Largest dequantisation cost per weight (instructions) that still hides behind the
    weight load (memory-bound) and behind the MMA at batch M (compute-bound): the two
    thresholds the paper derives in Sec. 3.3."""
    per_weight_ld = bytes_per_weight(4, group) / rates.mem_bytes_per_s
    per_weight_mma = min(m_tile, M) * 2.0 / rates.mma_ops_per_s
    return {"vs_load": per_weight_ld * rates.valu_lane_ops_per_s,
            "vs_mma": per_weight_mma * rates.valu_lane_ops_per_s}
