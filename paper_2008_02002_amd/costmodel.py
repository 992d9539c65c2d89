"""Operation and byte counts of the quantized scan, used for roofline accounting.

Two models live here:
  * the paper's own count (Section 3.4, Table 1), kept so the figures it prints in
    Section 5 can be reproduced from it;
  * the credited work this build reports against the MI355X rooflines: one XOR and
    one population count per (plane pair, 32-bit word), nothing else.
"""
from __future__ import annotations

# MI355X nominal ceilings.  The vector-integer figure is derived from unit counts:
# 256 compute units x 4 SIMDs x 16 lanes x 2.4 GHz, one 32-bit integer operation per
# lane per clock (no packed or dual-rate form exists for XOR or population count).
CU_COUNT = 256
CLOCK_HZ = 2.4e9
VALU_INT_LANE_OPS_PER_S = CU_COUNT * 4 * 16 * CLOCK_HZ      # 39.3e12
HBM_BYTES_PER_S = 8.0e12


def words32(d: int) -> int:
    return (d + 31) // 32


def table1_ops(d: int, bx: int, by: int) -> float:
    """Section 3.4, Table 1, quantized row: Bx*By*(d/64) XOR, as many POPCNT, and
    Bx*By*(d/64) - 1 shifts and as many additions."""
    t = bx * by * d / 64.0
    return 2 * t + 2 * (t - 1)


def table1_fp32_ops(d: int) -> float:
    """Section 3.4, Table 1, fp32 row: d multiplications and d - 1 additions."""
    return d + (d - 1)


def table1_bytes(d: int, bx: int, by: int) -> float:
    """Section 3.4, Table 1: (Bx + By)(d/64) 8-byte words for the two operands."""
    return (bx + by) * d / 64.0 * 8


def table1_fp32_bytes(d: int) -> float:
    return 2 * d * 4


def credited_lane_ops_per_pair(d: int, bq: int, bd: int) -> int:
    """XOR + population count per (query, database row): 2 * Bq * Bd * ceil(d/32)."""
    return 2 * bq * bd * words32(d)


def code_bytes_per_row(d: int, bits: int) -> int:
    """Stored bytes of one encoded row: bits planes of ceil(d/32) 32-bit words."""
    return 4 * bits * words32(d)


def encode_bytes_per_row(d: int, bits: int) -> int:
    """HBM traffic the encoder must move per row: the fp32 row in, its planes out."""
    return 4 * d + code_bytes_per_row(d, bits)
