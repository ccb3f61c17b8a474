"""Host-only checks of the benchmark's bookkeeping: the FLOP counts it prices kernels with, the
counter parser behind profiles/traffic.json and the abridged U-Net record of the one-line output."""
import csv
import io
import json
import os
import sys
from contextlib import redirect_stdout

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)
import bench  # noqa: E402


def test_exact_flop_count_is_the_number_of_in_bounds_multiply_adds():
    """2 N C_in C_out (3D-2)(3H-2)(3W-2) against a brute-force count of the taps that hit the volume."""
    for (n, d, h, w, ci, co) in [(1, 1, 1, 1, 1, 1), (2, 3, 4, 5, 3, 2), (1, 8, 8, 16, 4, 4)]:
        taps = 0
        for z in range(d):
            for y in range(h):
                for x in range(w):
                    for kd in (-1, 0, 1):
                        for kh in (-1, 0, 1):
                            for kw in (-1, 0, 1):
                                taps += 0 <= z + kd < d and 0 <= y + kh < h and 0 <= x + kw < w
        assert bench.conv_flops(n, d, h, w, ci, co) == 2.0 * n * ci * co * taps
    # nominal count (every tap) is 3.2 % higher at 64^3, as the documentation says
    assert abs(2.0 * 27 * 64 ** 3 * 32 * 32 / bench.conv_flops(1, 64, 64, 64, 32, 32) - 1.032) < 1e-3


def test_unet_flops_sum_the_program_calls():
    """The U-Net total the benchmark divides by is the sum over the step program's convolution calls
    (three passes per layer, no backward-data for the first), with exact instead of nominal counts."""
    from paper_1811_12174_amd.program import unet_program
    base, levels, n, s = 8, 3, 2, 16
    prog = unet_program(base, 1, levels, n, s, s, s)
    nominal = sum(c.flops for c in prog.calls if c.fn.startswith("conv_"))
    exact = bench.unet_flops(base, levels, n, s)
    assert 0.80 * nominal < exact < nominal
    layers = {c.layer for c in prog.calls if c.fn == "conv_fwd"}
    assert len(layers) == 2 * levels + 2 * (levels - 1)


def _counter_csv(path, counter, rows):
    with open(path, "w", newline="") as f:
        wr = csv.DictWriter(f, fieldnames=["Kernel_Name", "Counter_Name", "Counter_Value"])
        wr.writeheader()
        for name, value in rows:
            wr.writerow({"Kernel_Name": name, "Counter_Name": counter, "Counter_Value": value})


def test_traffic_parser_scales_by_the_calibration_kernel_and_keeps_other_entries(tmp_path):
    add = "void at::native::vectorized_elementwise_kernel<4, at::native::CUDAFunctorOnSelf_add<float>, std::array<char*, 2ul> >(int)"
    other = "void at::native::vectorized_elementwise_kernel<4, at::native::bfloat16_copy_kernel_cuda(at::TensorIteratorBase&)>"
    k = "void k3::conv_mfma_zs_kernel<0, false, false>(k3::MfmaParams)"
    known_kib = (64 << 20) * 4 / 1024.0
    f, w = str(tmp_path / "f.csv"), str(tmp_path / "w.csv")
    # the fetch counter reads half the bytes (as on the chip), the write counter all of them; a larger
    # elementwise kernel of another kind must not be taken for the calibration
    _counter_csv(f, "FETCH_SIZE", [(add, known_kib / 2), (add, known_kib / 2), (other, 10 * known_kib), (k, 1000.0), (k, 3000.0)])
    _counter_csv(w, "WRITE_SIZE", [(add, known_kib), (other, 10 * known_kib), (k, 500.0)])
    out = str(tmp_path / "traffic.json")
    with open(out, "w") as fh:
        json.dump({"kept": {"x": 1}}, fh)
    with redirect_stdout(io.StringIO()):
        bench.pmc_parse(f, w, key="case", path=out)
    t = json.load(open(out))
    assert t["kept"] == {"x": 1}
    assert abs(t["_calibration"]["case"]["fetch_scale"] - 2.0) < 1e-9 and abs(t["_calibration"]["case"]["write_scale"] - 1.0) < 1e-9
    rec = t["case"]["conv_mfma_zs_kernel"]
    assert rec["fetch_bytes"] == round(2000.0 * 1024 * 2.0) and rec["write_bytes"] == round(500.0 * 1024)
    assert rec["bytes_per_launch"] == rec["fetch_bytes"] + rec["write_bytes"]


def test_abridged_unet_record_keeps_the_metric_and_drops_the_plan_listings():
    leg = {"ms_per_step": 350.0, "voxels_per_s": 9.6e7, "overhead_pct": 170.0, "ms_copies_only": 312.0, "overlap_fraction": 0.7,
           "achieved_gbs_out": 56.8, "achieved_gbs_in": 56.9, "achieved_pct_of_one_direction_peak": 99.7,
           "copies_only_pct_of_link": 58.0, "accounted_peak_gb": 25.8, "device_budget_gb": 26.0,
           "no_swap_under_budget": "refused: device budget exceeded at call 18", "swap_under_budget": "completed",
           "bytes_out_per_step": 8858370048, "bytes_in_per_step": 8858370048,
           "plan": {"swapped_tensors": ["a1_0", "a2_0", "b:a1_0"], "predicted_ms": 355.0, "prefetch_lead_calls": [1, 2, 3]}}
    u = {"workload": "cfg4", "steps": 2, "ms_per_step_no_swap": 129.0, "voxels_per_s_no_swap": 2.6e8, "conv_tflops_no_swap": 1289.0,
         "pct_mfma_peak_no_swap": 51.2, "accounted_peak_gb_no_swap": 34.6, "link_gbs": {"d2h_alone": 56.0},
         "weight_update_ms": 0.4, "planned_for_budget": leg}
    c = bench.compact_unet(u)
    assert c["ms_per_step_no_swap"] == 129.0 and c["link_gbs"] == {"d2h_alone": 56.0} and "weight_update_ms" not in c
    p = c["planned_for_budget"]
    assert p["voxels_per_s"] == 9.6e7 and p["overlap_fraction"] == 0.7 and p["no_swap_under_budget"] == "refused"
    assert p["gb_out"] == 8.86 and p["tensors_swapped"] == 3 and p["predicted_ms"] == 355.0 and "plan" not in p
    assert len(json.dumps(c)) < 1200
