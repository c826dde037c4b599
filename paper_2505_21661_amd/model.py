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


# ---- overlap models of Table 4 (Sec. 5.2 "Performance Modeling for GPU Overlapping") -----------------
#
# The models work on stage latencies: T_load^i and T_comp^i of pipeline stage i, as the stage table
# of kp_pairs_stages gives them (slowest wave per workgroup, region and iteration).  The table in
# the paper is partly damaged; the readings taken are stated with each function.

def swp_discriminant(t_load, t_comp, n_wg: int, n_pipe: int) -> float:
    """Delta of the software-pipelining model: N_WG * N_pipe * sum_i T_comp^i - max_i (T_load^i + T_comp^i).

    Delta >= 0: the computation of all resident warp groups and pipeline stages covers the slowest
    load + compute stage, so loading is hidden.  Read from the first line of the model as printed."""
    assert len(t_load) == len(t_comp) and len(t_comp) > 0
    return n_wg * n_pipe * float(sum(t_comp)) - max(l + c for l, c in zip(t_load, t_comp))


def swp_latency(t_load, t_comp, n_loop: int, n_pipe: int, n_wg: int = 1) -> float:
    """Software-pipelining model: sum_i T_comp^i * N_loop when Delta >= 0 (loads fully overlapped),
    else max_i (T_load^i + T_comp^i) * N_loop / N_pipe (the slowest stage dominates, N_pipe of them in flight)."""
    if swp_discriminant(t_load, t_comp, n_wg, n_pipe) >= 0:
        return float(sum(t_comp)) * n_loop
    return max(l + c for l, c in zip(t_load, t_comp)) * n_loop / n_pipe


def ws_latency(stage_latency, critical_path) -> float:
    """Warp-specialisation model: the sum of the latencies of the stages on the critical path."""
    return float(sum(stage_latency[i] for i in critical_path))


def compute_time(flops: float, throughput: float) -> float:
    """Compute model: FLOPs / throughput."""
    return flops / throughput


def memory_time(t_read: float, n_bytes: float, bandwidth: float) -> float:
    """Memory model: T_read + bytes / bandwidth (a fixed read latency plus the transfer)."""
    return t_read + n_bytes / bandwidth


def stage_latencies(table, wg: int, n_iter: int | None = None):
    """Mean latency per region of one workgroup over its first n_iter iterations (all that ran if None),
    from a parsed stage table (binding.parse_stages): the T^i the models above take."""
    out = []
    for r in range(table.shape[1]):
        row = table[wg, r]
        ran = row["n_waves"] > 0
        if n_iter is not None:
            ran[n_iter:] = False
        out.append(float(row["max_dur"][ran].mean()) if ran.any() else 0.0)
    return out


def critical_stage_per_iteration(table, wg: int):
    """For every iteration of one workgroup, the region whose stage lasted longest (-1 where none ran):
    the stage a critical-path analysis looks at first (Sec. 3.3 "Critical-path Analysis")."""
    t = table[wg]
    dur = t["max_dur"].astype("int64")
    dur[t["n_waves"] == 0] = -1
    best = dur.argmax(axis=0)
    best[dur.max(axis=0) < 0] = -1
    return best
