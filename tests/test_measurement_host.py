"""Host-side logic of the measurement helpers (no GPU): the ratios derived from raw rocprofv3 counters, the ideal
sparse / dense ratios quoted by the bench line, the refusal of a run on more than one GPU, and that the hardware probe
program still compiles for gfx950."""
import os
import re
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_counter_ratios_follow_from_their_definitions():
    from paper_2305_10727_amd.profiling import derived
    # a made-up launch of 1000 shader clocks on a chip of 1024 SIMDs / 32 shader engines in which every SIMD issues 10
    # matrix instructions (16 clocks of matrix pipe each) and 50 other vector instructions
    simds, clocks, mfma, valu = 1024, 1000.0, 10, 50
    c = {
        "SQ_BUSY_CYCLES": clocks * 32,
        "SQ_WAVES": 2048.0,
        "SQ_WAVE_CYCLES": 2048.0 * 900.0 / 4.0,              # every wavefront lives 900 clocks, counted in units of 4
        "SQ_INSTS_MFMA": float(simds * mfma),
        "SQ_VALU_MFMA_BUSY_CYCLES": float(simds * mfma * 16),
        "SQ_INSTS_VALU": float(simds * (valu + mfma)),        # the counter includes the matrix instructions
        "SQ_ACTIVE_INST_VALU": float(simds * (valu + 4 + mfma)),
        "SQ_LDS_IDX_ACTIVE": 256 * 250.0,
        "SQ_LDS_BANK_CONFLICT": 256 * 25.0,
        "SQ_WAIT_INST_ANY": 2048.0 * 90.0,
    }
    d = derived(c)
    get = lambda start: [v for k, v in d.items() if k.startswith(start)][0]
    assert get("launch_clocks") == clocks
    assert get("mean wavefront lifetime") == 900.0
    assert get("mfma_util =") == pytest.approx(mfma * 16 / clocks)
    assert get("vector instructions (matrix ones excluded)") == pytest.approx(valu / clocks)
    assert get("valu_util =") == pytest.approx(2.6 * valu / clocks)
    assert get("mfma_util + valu_util") == pytest.approx((mfma * 16 + 2.6 * valu) / clocks)
    assert get("lds_util") == pytest.approx(0.25)
    assert get("other vector instructions per matrix instruction") == pytest.approx(valu / mfma)
    assert get("lds_bank_conflict") == pytest.approx(0.1)
    assert get("wait_inst_any") == pytest.approx(0.4)
    assert get("mfma_busy_cycles / mfma_insts") == 16.0
    # without the busy counter the dispatch-active counter of the 8 dies is the (longer) fallback
    d2 = derived({"GRBM_GUI_ACTIVE": 8 * 1300.0, "SQ_VALU_MFMA_BUSY_CYCLES": c["SQ_VALU_MFMA_BUSY_CYCLES"]})
    assert [v for k, v in d2.items() if k.startswith("launch_clocks")] == [1300.0]


def test_ideal_ratios_quoted_by_the_bench_line():
    """both sides on their own roofline at the nominal peaks: on c1 INT8 the sparse side is bound by HBM (the Y write),
    the dense side, by a hair, by the matrix pipe; c1 FP16 is bound by the matrix pipe on both sides"""
    from paper_2305_10727_amd.report import ideal_speedup
    M, K, N = 12608, 768, 3072
    i8, f16 = ideal_speedup(M, K, N, "int8"), ideal_speedup(M, K, N, "fp16")
    io = M * K + 8 * N + 2 * M * N
    ops = 2.0 * M * N * K
    assert ops / 5035e12 > (io + N * K) / 8e12 and ops / 10070e12 < (io + N * K // 2 + N * K // 8) / 8e12
    assert i8 == pytest.approx((ops / 5035e12) / ((io + N * K // 2 + N * K // 8) / 8e12))
    assert f16 == pytest.approx(5030.0 / 2515.0 * (ops / 5030e12) / max(ops / 5030e12, (M * K * 2 + 8 * N + 2 * M * N + N * K + N * K // 8) / 8e12))
    src = open(os.path.join(ROOT, "bench.py")).read()
    quoted = {k: float(v) for k, v in re.findall(r'"(int8|fp16)_ideal_speedup_vs_dense": ([0-9.]+)', src)}
    assert quoted == {"int8": pytest.approx(i8, abs=0.01), "fp16": pytest.approx(f16, abs=0.01)}
    # long K, few channels: matrix-bound on both sides, the full factor of two
    assert ideal_speedup(65792, 5120, 1280, "int8") == pytest.approx(2.0, abs=0.01)


def test_bench_refuses_more_than_one_gpu():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=300)
    assert res.returncode != 0 and res.stdout.strip() == ""
    assert "--gpus 1" in res.stderr


def test_probe_program_compiles_for_gfx950(tmp_path):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(hipcc):
        pytest.skip("no hipcc")
    src = os.path.join(ROOT, "paper_2305_10727_amd", "probes", "hw_probes.hip")
    res = subprocess.run([hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                          "-c", src, "-o", str(tmp_path / "hw_probes.o")], capture_output=True, text=True, timeout=900)
    assert res.returncode == 0, res.stderr[-2000:]
