"""The paper's overhead model (Sec. 5.4 "Optimization Degradation", eq. (1)).

    T_theoretical = T_vanilla + N_record * Cycle_record

N_record is the number of records one wave writes, Cycle_record the measured cost of one record
(the calibration kernel's empty region gives the cost of a START/END pair).  The paper compares the
model with the measured time of the instrumented kernel (Table 5: within 2 %).
"""
from __future__ import annotations


def theoretical_ticks(t_vanilla: float, n_record: int, cycle_record: float) -> float:
    return t_vanilla + n_record * cycle_record


def relative_performance(t_vanilla: float, t_theoretical: float, t_actual: float) -> tuple[float, float, float]:
    """The three entries of the paper's "relative performance" row: each time over the model's."""
    return t_vanilla / t_theoretical, 1.0, t_actual / t_theoretical
