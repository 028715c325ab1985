"""Host logic of the measurement tools, without a GPU: the byte accountings of bench.py, its refusal of
more than one GPU, the traffic table's source stamp, and the summaries made from profiler CSV files."""
import csv
import importlib.util
import io
import os
import subprocess
import sys
from contextlib import redirect_stdout

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def load_bench():
    spec = importlib.util.spec_from_file_location("bench_under_test", os.path.join(ROOT, "bench.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_stage_bytes_follow_the_passes_of_the_design():
    B = load_bench()
    p_w, p_o, nbits = 0.25, 0.125, 4
    s = p_w + 2 * p_o                                      # survivor values per parameter: 0.5
    st = B.stage_bytes_per_param(p_w, p_o, nbits, 10)
    assert st["stats_stream"] == 12.0                      # W_prev, W, m read once
    assert st["mask_slots"] == 16.0 + 0.125 + 4.0 * s      # four arrays read, bitmap and survivor slots written
    assert st["mask_gather"] == 8.0 * s + 0.25 * p_w
    assert st["km_bucket_stats"] == 4.0 * s and st["km_scatter"] == 8.0 * s and "km_count" not in st
    assert st["assign_pack"] == 4.0 * s + s * nbits / 8.0
    assert st["decode_main"] == 8.0 + 0.125 * (1 + p_w) + s * nbits / 8.0
    # 16-bit weights: only the passes over W_prev, W and W_hat shrink
    h = B.stage_bytes_per_param(p_w, p_o, nbits, 10, wb=2.0)
    assert h["stats_stream"] == 8.0 and h["mask_slots"] == st["mask_slots"] - 4.0
    assert h["decode_main"] == st["decode_main"] - 4.0 and h["km_scatter"] == st["km_scatter"]


def test_survey_formula():
    B = load_bench()
    assert B.survey_bytes_per_param(0.0, 0.0) == pytest.approx(40.2)
    assert B.survey_bytes_per_param(0.3, 0.1) == pytest.approx(32.2 + 58.5 * 0.5 + 8.0)
    assert B.survey_bytes_per_param(0.3, 0.1, wb=2.0) == pytest.approx(32.2 - 8.0 + 58.5 * 0.5 + 4.0)


def test_stage_kernel_names_exist_in_the_sources():
    B = load_bench()
    src = ""
    csrc = os.path.join(ROOT, "paper_2406_11257_amd", "csrc")
    for name in os.listdir(csrc):
        if name.endswith(".hip"):
            src += open(os.path.join(csrc, name)).read()
    for weights in ("f32", "bf16"):
        for kernel in B.stage_kernels(weights).values():
            assert f"void {kernel.split('<')[0]}(" in src, kernel


def test_traffic_table_is_used_only_with_the_sources_it_was_measured_on(tmp_path, monkeypatch):
    B = load_bench()
    from paper_2406_11257_amd.rocprof_summary import sources_hash
    prof = tmp_path / "profiles"
    prof.mkdir()
    monkeypatch.setattr(B, "ROOT", str(tmp_path))
    (prof / "hbm_traffic.txt").write_text(f"# comment\nsources {sources_hash()}\n"
                                          "traffic llama-7b k_a<false> 1000 200\ntraffic other k_a<false> 5 5\n")
    table, fresh = B.measured_traffic("llama-7b")
    assert fresh and table == {"k_a<false>": (1000.0, 200.0)}
    (prof / "hbm_traffic.txt").write_text("sources 0123456789abcdef\ntraffic llama-7b k_a<false> 1000 200\n")
    table, fresh = B.measured_traffic("llama-7b")
    assert not fresh and table                             # the table is read, and reported as stale
    (prof / "hbm_traffic.txt").unlink()
    assert B.measured_traffic("llama-7b") == ({}, False)


def test_committed_traffic_table_is_well_formed():
    lines = open(os.path.join(ROOT, "profiles", "hbm_traffic.txt")).read().splitlines()
    stamps = [l.split()[1] for l in lines if l.startswith("sources ")]
    rows = [l.split() for l in lines if l.startswith("traffic ")]
    assert len(stamps) == 1 and len(stamps[0]) == 16 and int(stamps[0], 16) >= 0
    assert rows and all(len(r) == 5 and float(r[3]) >= 0 and float(r[4]) >= 0 for r in rows)
    assert any(r[2] == "k_copy_probe" and abs(float(r[3]) - 2 ** 30) < 2 ** 20 for r in rows)   # the calibration itself


def write_csv(path, header, rows):
    os.makedirs(os.path.dirname(path), exist_ok=True)
    with open(path, "w", newline="") as f:
        w = csv.writer(f)
        w.writerow(header)
        w.writerows(rows)


def test_summaries_from_profiler_csv(tmp_path):
    from paper_2406_11257_amd import rocprof_summary as R
    assert R.short("void (anonymous namespace)::k_mask_slots<false, true>(Workspace, GroupParams)") == "k_mask_slots<false,true>"
    assert R.short("at::native::vectorized_elementwise_kernel<4>") is None
    d = str(tmp_path / "stats")
    write_csv(d + "/x/1_kernel_trace.csv", ["Kernel_Name", "Start_Timestamp", "End_Timestamp"],
              [["k_a(Workspace)", 0, 2_000_000], ["k_a(Workspace)", 10, 4_000_010], ["k_b<4u>(int)", 0, 1_000_000],
               ["some_torch_kernel", 0, 9_000_000]])
    out = io.StringIO()
    with redirect_stdout(out):
        R.stats(d)
    text = out.getvalue().splitlines()
    a = [l for l in text if l.startswith("k_a ")][0].split()
    assert a[1] == "2" and float(a[2]) == 6.0 and float(a[3]) == 3.0 and float(a[4]) == 2.0 and float(a[5]) == 4.0
    assert [l for l in text if l.startswith("all library kernels")][0].split()[-2:] == ["3", "7.000"]
    assert not any("torch" in l for l in text)

    # counters: KiB per dispatch, scaled by what the copy probe reads for its known 1 GiB
    f, w = str(tmp_path / "fetch"), str(tmp_path / "write")
    hdr = ["Dispatch_Id", "Kernel_Name", "Counter_Name", "Counter_Value"]
    write_csv(f + "/y/1_counter_collection.csv", hdr,
              [[1, "k_copy_probe(void*)", "FETCH_SIZE", 524288], [2, "k_a(Workspace)", "FETCH_SIZE", 1000], [3, "k_a(Workspace)", "FETCH_SIZE", 3000]])
    write_csv(w + "/y/1_counter_collection.csv", hdr,
              [[1, "k_copy_probe(void*)", "WRITE_SIZE", 1048576], [2, "k_a(Workspace)", "WRITE_SIZE", 10], [3, "k_a(Workspace)", "WRITE_SIZE", 30]])
    out = io.StringIO()
    with redirect_stdout(out):
        R.traffic("wl", f, w)
    lines = out.getvalue().splitlines()
    assert f"sources {R.sources_hash()}" in lines
    row = [l.split() for l in lines if l.startswith("traffic wl k_a ")][0]
    assert float(row[3]) == 2000 * 2.0 * 1024 and float(row[4]) == 20 * 1.0 * 1024
    with pytest.raises(SystemExit):
        R.stats(str(tmp_path / "nothing"))
