"""Host-side arithmetic of bench.py (no GPU): the algorithmic work per launch that the roofline
figures divide by, the choice of the dominant kernel, the parsing of the counter summaries."""
import importlib.util
import os

import pytest

from paper_2003_03477_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
spec = importlib.util.spec_from_file_location("bench", os.path.join(ROOT, "bench.py"))
bench = importlib.util.module_from_spec(spec)
spec.loader.exec_module(bench)


def test_algorithmic_bytes_match_the_per_unit_figures():
    mid, large = synth.mid(), synth.large()
    n_mid = mid.batch * mid.num_tables * 21            # mean ids per step: B*T*(lambda+1)
    assert n_mid == 344064
    # gather: 260 B per id (256-byte row + index) and per bag (pooled vector + offset)
    assert bench.hbm_bytes("gather", mid, n_mid, 0) == n_mid * 260 + 2048 * 8 * 260
    assert abs(bench.hbm_bytes("gather", mid, n_mid, 0) / 1e6 - 93.7) < 0.1
    n_large = large.batch * large.num_tables * 31
    assert abs(bench.hbm_bytes("gather", large, n_large, 0) / 1e9 - 1.772) < 0.001
    # row update: per occurrence a gradient row and a sorted pair, per distinct row the row
    # and its accumulator read and written; all-distinct upper bound of the Mid config
    assert bench.hbm_bytes("row_update_chunk", mid, n_mid, n_mid) == n_mid * (264 + 520)
    # interaction backward: df row + V tile read + dV tile written per sample
    F = 64 + 8 * 9 // 2
    assert bench.hbm_bytes("interaction_bwd", mid, 0, 0) == 2048 * (4 * F + 2 * 9 * 256)
    with pytest.raises(KeyError):
        bench.hbm_bytes("nope", mid, 0, 0)


def test_mlp_flops_of_the_configs():
    flops, first_top = bench.mlp_flops(synth.large())
    assert first_top == 3
    per_sample_fwd = 2 * (13 * 512 + 512 * 256 + 256 * 64 + 415 * 1024 + 1024 * 1024 + 1024 * 512 + 512 * 256)
    assert flops["mlp_fwd"] == 8192 * per_sample_fwd
    assert flops["mlp_wgrad"] == flops["mlp_fwd"]
    assert flops["mlp_dgrad"] == flops["mlp_fwd"] - 8192 * 2 * 13 * 512     # no data gradient for the input
    total = sum(flops.values())
    assert 110e9 < total < 114e9                                             # about 112 GFLOP per Large step
    mid_total = sum(bench.mlp_flops(synth.mid())[0].values())
    assert 2.7e9 < mid_total < 2.9e9


def test_dominant_kernel_is_the_largest_per_step_time_over_all_classes():
    """Classes are ranked by launches per step x duration with one stream active (the event
    brackets under several streams inflate short launches); without that figure, by the
    in-region brackets."""
    kernels = {
        "gather": {"total_ms_in_timed_region": 5.0, "bound": "hbm", "GBps": 4000.0, "frac_of_hbm_peak": 0.5,
                   "avg_us": 100.0, "alone_avg_us": 90.0, "brackets": 50, "launches_per_step": 1,
                   "algorithmic_bytes_per_launch": 4e8, "counter_bytes_per_launch": 2e8},
        "mlp_fwd": {"total_ms_in_timed_region": 9.0, "bound": "mfma", "TFLOPps": 300.0,
                    "frac_of_bf16_mfma_peak": 0.12, "alone_frac_of_bf16_mfma_peak": 0.3,
                    "avg_us": 50.0, "alone_avg_us": 20.0, "brackets": 350,
                    "launches_per_step": 7, "algorithmic_flops_per_launch": 6e9},
        "sort_all_passes": {"avg_us": 200.0, "brackets": 8},      # a group class: not a candidate
    }
    r = bench.pick_roofline(kernels, 8)      # 7 x 20 us against 1 x 90 us
    assert r["kernel"] == "mlp_fwd" and r["bound"] == "mfma" and r["peak"] == 2500.0
    assert r["unit"] == "TFLOP/s" and r["frac"] == 0.12 and r["traffic"] is None
    assert r["ranking_us_per_step_one_stream"] == {"gather": 90.0, "mlp_fwd": 140.0}
    kernels["mlp_fwd"]["alone_avg_us"] = 10.0   # 70 us per step: the gather leads, although the
    r = bench.pick_roofline(kernels, 8)         # in-region brackets sum to more for the MLP
    assert r["kernel"] == "gather" and r["peak"] == 8000.0 and r["traffic"] == 2e8
    assert r["largest_mfma_class"]["kernel"] == "mlp_fwd" and r["largest_mfma_class"]["frac"] == 0.12
    del kernels["mlp_fwd"]["alone_avg_us"]      # no one-stream figure: 7 x 50 us of brackets
    assert bench.pick_roofline(kernels, 8)["kernel"] == "mlp_fwd"
    assert bench.pick_roofline({"sort_all_passes": {"avg_us": 1.0}}, 1) is None


def test_counter_summaries_are_parsed():
    for wl in ("large", "mid"):
        for k in ("gather", "row_update_chunk", "interaction_bwd"):
            v = bench.measured_traffic(wl, k)
            assert v is not None and v > 1e6, (wl, k)
        for k in ("gather", "row_update_chunk", "mlp_fwd", "mlp_dgrad", "mlp_wgrad"):
            v = bench.profiler_in_region_us(wl, k)
            assert v is not None and 1.0 < v < 1e4, (wl, k)
    assert bench.profiler_in_region_us("large", "no_such_kernel") is None
    assert bench.measured_traffic("large", "no_such_kernel") is None
    assert bench.measured_traffic("no_such_workload", "gather") is None


def test_worker_lists():
    assert bench.parse_workers("2", 4) == [2, 2, 2, 2]
    assert bench.parse_workers("8,1,1,1", 4) == [8, 1, 1, 1]


def test_fractions_of_the_measured_copy_ceiling():
    out = {"roofline": {"bound": "hbm", "achieved": 2500.0, "alone_achieved": 4000.0},
           "kernels": {"gather": {"bound": "hbm", "GBps": 3000.0, "alone_GBps": 4500.0},
                       "mlp_fwd": {"bound": "mfma", "TFLOPps": 300.0},
                       "sort_all_passes": {"avg_us": 1.0}},
           "secondary": {"mid": {"roofline": {"bound": "mfma", "achieved": 30.0},
                                 "kernels": {"row_update_chunk": {"bound": "hbm", "GBps": 1000.0}}}}}
    bench.annotate_copy_ceiling(out, 5000.0)
    assert out["roofline"]["frac_of_copy_ceiling"] == 0.5 and out["roofline"]["alone_frac_of_copy_ceiling"] == 0.8
    assert out["kernels"]["gather"]["frac_of_copy_ceiling"] == 0.6
    assert out["kernels"]["gather"]["alone_frac_of_copy_ceiling"] == 0.9
    assert "frac_of_copy_ceiling" not in out["kernels"]["mlp_fwd"]
    assert "frac_of_copy_ceiling" not in out["secondary"]["mid"]["roofline"]
    assert out["secondary"]["mid"]["kernels"]["row_update_chunk"]["frac_of_copy_ceiling"] == 0.2
