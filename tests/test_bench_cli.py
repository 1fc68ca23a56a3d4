"""Host-side contract of bench.py that needs no GPU: one GPU only, and the product never imports the oracle."""
import os
import re
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0 and "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_the_product_package_never_imports_the_oracle():
    pkg = os.path.join(ROOT, "paper_2604_02047_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f), encoding="utf-8").read()
                assert not re.search(r"^\s*(from|import)\s+oracle\b", text, re.M), f
                assert "goose_oracle" not in text and "goose_draft" not in text, f


def test_bench_uses_the_oracle_only_for_the_cpu_baseline():
    text = open(os.path.join(ROOT, "bench.py"), encoding="utf-8").read()
    uses = [m.start() for m in re.finditer(r"^\s*(from|import)\s+oracle\b", text, re.M)]
    assert len(uses) == 1 and uses[0] > text.index("def cpu_baseline(")


def test_counter_figures_are_reported_only_for_the_sources_they_were_recorded_for(tmp_path, monkeypatch):
    """roofline.traffic and counter_GB_per_step come from a committed profiler summary; a summary recorded
    for other sources (another hash over csrc/ and goose.h) must read as null, with the reason."""
    sys.path.insert(0, ROOT)
    import bench
    from paper_2604_02047_amd.profiling import source_hash
    body = ("recorded 2026-01-01 for the library sources with hash {h}\n"
            "last step of the run: 265 launches, fetch 15000.00 MB, write 800.00 MB\n"
            "kernel  wgs_x gy n avg_us fetch_MB write_MB\n"
            "k_gemm_bf16<2, 4, 1, 1, false, true>   256 1 704 33.7 184.60 1.41\n"
            "k_gemm_bf16<2, 4, 1, 0, false, true>   128 2 704 20.0 104.92 6.29\n")
    (tmp_path / "profiles").mkdir()
    monkeypatch.setattr(bench, "ROOT", str(tmp_path))
    f = tmp_path / "profiles" / "traffic_w.txt"
    f.write_text(body.format(h=source_hash()))
    rec = bench.recorded_traffic("w")
    assert rec["gate_up_bytes"] == 186010000 and rec["step_bytes"] == 15800000000 and "NOT" not in rec["source"]
    f.write_text(body.format(h="0123456789ab"))
    rec = bench.recorded_traffic("w")
    assert rec["gate_up_bytes"] is None and rec["step_bytes"] is None and "NOT this build" in rec["source"]
    assert bench.recorded_traffic("absent") == {"gate_up_bytes": None, "step_bytes": None, "source": None}
