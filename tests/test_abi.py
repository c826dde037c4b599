"""The C ABI library builds, loads and exports every entry point that include/kperf.h declares
(no GPU needed; no compute calls are made)."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "kperf.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"\b(kp_[a-z_0-9]+)\s*\(", text)
    return sorted(set(names))


def test_header_declares_the_named_entry_points():
    names = declared_symbols()
    for must in ("kp_gemm_instrumented", "kp_attn_instrumented", "kp_trace_reduce", "kp_calibrate",
                 "kp_trace_bytes", "kp_stats_bytes", "kp_last_error", "kp_trace_pairs", "kp_trace_waits", "kp_pairs_stages"):
        assert must in names


def test_library_exports_every_declared_symbol():
    import paper_2505_21661_amd as kp
    from paper_2505_21661_amd import build as kbuild

    if not os.path.exists(kp.binding.LIB_PATH):
        kbuild.build()
    lib = ctypes.CDLL(kp.binding.LIB_PATH)
    for name in declared_symbols():
        assert hasattr(lib, name), f"libkperf.so does not export {name}"


def test_size_helpers_and_struct_sizes():
    import paper_2505_21661_amd as kp

    assert ctypes.sizeof(kp.binding.kp_trace_hdr) == 64
    # header + workgroup headers + 8-byte records
    assert kp.kp_trace_bytes(64, 4, 512) == 64 + 128 * 64 + 8 * 64 * 512
    assert kp.kp_trace_bytes(1, 2, 64) - kp.kp_trace_bytes(1, 2, 0) == 512   # 64 slots = 0.5 KB (Sec. 4.2)
    assert kp.kp_trace_bytes(1, 3, 64) == 0 and kp.kp_trace_bytes(1, 17, 68) == 0
    R, n_wg, W = 5, 7, 4
    assert kp.kp_stats_bytes(n_wg, W, R) == 128 + 8 * (64 * R + 5 * R + 2 * R * R) + 16 * n_wg * W * R
    assert kp.kp_stats_bytes(1, 0, 3) == 0
    # count array padded to 16 bytes + 16-byte rows, cap_wave / 2 per (workgroup, wave)
    assert kp.kp_pairs_bytes(3, 2, 64) == 32 + 16 * 3 * 2 * 16
    assert kp.kp_pairs_bytes(1, 3, 64) == 0
    # 16 header words, 64-bin histogram and 7 totals per region, 16 bytes per (workgroup, wave, region)
    assert kp.kp_waits_bytes(n_wg, W, R) == 128 + 8 * (64 * R + 7 * R) + 16 * n_wg * W * R
    assert kp.kp_waits_bytes(1, 17, 3) == 0 and kp.kp_waits_bytes(1, 4, 129) == 0
    # 4 header words, 16 bytes per (workgroup, region, iteration)
    assert kp.kp_stages_bytes(n_wg, R, 10) == 32 + 16 * n_wg * R * 10 and kp.kp_stages_bytes(1, 3, 0) == 0
    assert ctypes.sizeof(ctypes.c_uint32) * 4 == 16  # kp_stage_row and kp_pair_row are four u32
    assert kp.kp_last_error() == "" or isinstance(kp.kp_last_error(), str)


def test_host_side_argument_checks_need_no_gpu():
    """Shape queries and argument validation run on the host before any HIP call."""
    import paper_2505_21661_amd as kp

    assert kp.kp_gemm_launch_shape(256, 256, 256) == (16, 4, 3)
    assert kp.kp_gemm_launch_shape(4096, 4096, 4096) == (256, 8, 4)
    assert kp.kp_attn_launch_shape(4, 32, 4096, 128) == (4096, 4, 3)
    import pytest

    with pytest.raises(kp.KperfError) as e:
        kp.kp_gemm_launch_shape(100, 64, 32)
    assert e.value.status == kp.KP_ERR_UNSUPPORTED_SHAPE and "multiples" in str(e.value)
    with pytest.raises(kp.KperfError):
        kp.kp_attn_launch_shape(1, 1, 4096, 64)


def test_overhead_model_against_table_5(paper_values):
    """Eq. (1): T_theoretical = T_vanilla + N_record * Cycle_record, with the numbers of Table 5."""
    from paper_2505_21661_amd import model

    pv = paper_values
    t_vanilla, t_theoretical, t_actual = (pv[f"table5.active_cycles.{k}"] for k in ("vanilla", "theoretical", "actual"))
    # the table's model column is the vanilla column plus records x cycles: 25600 cycles of records
    extra = t_theoretical - t_vanilla
    assert extra == 25600
    assert model.theoretical_ticks(t_vanilla, 800, extra / 800) == t_theoretical
    rel = model.relative_performance(t_vanilla, t_theoretical, t_actual)
    assert [round(x, 2) for x in rel] == [pv[f"table5.relative_performance.{k}"] for k in ("vanilla", "theoretical", "actual")]
    assert round((t_actual - t_vanilla) / t_vanilla * 100, 1) == 15.2   # the GEMM's overhead in per cent


def test_layout_constants_match_the_paper(paper_values):
    import paper_2505_21661_amd as kp

    pv = paper_values
    assert ctypes.sizeof(ctypes.c_uint32) * 2 == pv["layout.record_bytes"]
    assert kp.kp_trace_bytes(1, 2, pv["layout.example_slots"]) - kp.kp_trace_bytes(1, 2, 0) == pv["layout.example_bytes"]
    assert pv["layout.example_slots"] // 2 == pv["layout.example_slots_per_group"]
