"""bench.py's command-line contract: the parts that can be checked without a GPU, and (on a GPU)
the shape of the JSON line on the small end of the workloads."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "ONE GPU" in r.stderr and r.stdout.strip() == ""


@pytest.mark.gpu
def test_json_line_has_the_contract_fields():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--workload", "wan21_14b", "--steps", "2",
                        "--warmup", "1", "--dense-reps", "1"], capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 2 and d["warmup"] == 1 and d["dtype"] == "bf16"
    assert d["config"]["workload"] == "wan21_14b" and "model" not in d["config"]
    rf = d["roofline"]
    assert rf["bound"] == "mfma" and rf["unit"] == "TFLOP/s" and abs(rf["frac"] - rf["achieved"] / rf["peak"]) < 1e-9
    cb = d["cpu_baseline"]
    assert cb["kind"] == "oracle" and cb["cores"] >= 1 and cb["value"] > 0 and cb["sample"]
    assert d["value"] > 0 and abs(d["ms_per_step"] - d["ms_per_layer"]) < 1e-9
    assert d["fp8"]["roofline"]["peak"] == 5000.0 and d["qk_norm_rope"]["roofline"]["bound"] == "hbm"
    # measured ceilings of the same box, live: zeros > random operands > with the kernel's instruction mix > the kernel
    assert rf["measured_peak_constant_operands"] > rf["measured_peak"] > rf["measured_peak_with_kernel_instruction_mix"] > rf["achieved"]
    assert cb["host_cpus"] >= 1 and cb["cores"] >= 1 and rf["traffic_live"] in (False, None)
    # the LDS of a compute unit, live: conflict-free reads far above the staging writes, the swizzle worth > 2x
    lr = rf["lds_rates"]
    assert lr["k_operand_ds_read_b128"]["bytes_per_clock_per_cu"] > 150 > lr["staging_ds_write_b128"]["bytes_per_clock_per_cu"]
    assert lr["vt_operand_ds_read_b64_tr_b16_swizzled_rows"]["bytes_per_clock_per_cu"] > 2 * lr["vt_operand_ds_read_b64_tr_b16_plain_rows"]["bytes_per_clock_per_cu"]


@pytest.mark.gpu
def test_matrix_core_rate_probe_runs_and_counts_its_work():
    import torch
    import paper_2502_01776_amd as S
    ops = torch.randn(1 << 19, device="cuda").to(torch.bfloat16)
    sink = torch.zeros(64 * 256, dtype=torch.float32, device="cuda")
    for form in (0, 1, 2):
        flop = S.svg_probe_mfma_bf16(form, 64, 10, ops, sink)
        torch.cuda.synchronize()
        assert flop == 64 * 4 * 10 * 16 * 2.0 * 32 * 32 * 16
        assert torch.isfinite(sink).all()


@pytest.mark.gpu
def test_lds_rate_probe_shows_what_the_swizzle_is_for():
    """The LDS probe times the operand reads of the attention kernels on one compute unit: with two
    wavefronts per SIMD the transposing read of the swizzled V tile must be conflict-free (a few clocks
    per wave instruction) and clearly faster than the same read on plain row-major rows."""
    import torch
    import paper_2502_01776_amd as S
    scratch = torch.zeros(16 + 512, dtype=torch.int64, device="cuda")
    clocks = {}
    for form in (0, 1, 2, 3):
        S.svg_probe_lds(form, 8, 200, scratch)          # warm-up
        S.svg_probe_lds(form, 8, 2000, scratch)
        torch.cuda.synchronize()
        t = scratch[:8].cpu().numpy()
        assert (t > 0).all()
        clocks[form] = float(t.max()) / (2000 * 16) / 8          # CU clocks per wave instruction
    assert clocks[1] < 4.5 and clocks[2] > 1.8 * clocks[1], clocks
    assert clocks[0] < 8.0 and clocks[3] > clocks[0], clocks

