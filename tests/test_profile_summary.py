"""Host logic of the profile summariser: which kernel's counters become bench.py's
`roofline.traffic`, and how they are scaled by the calibration copy."""
import csv
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

SPARSE = "void losa::attn_mfma_kernel<128, 16, 3, true, 2, 4, false>(losa::AttnPrepared, int)"
MANY_ROWS = "void losa::attn_mfma_kernel<128, 16, 2, false, 2, 8, true>(losa::AttnPrepared, int)"
COPY = "losa::calibration_copy_kernel(HIP_vector_type<unsigned int, 4u> const*, HIP_vector_type<unsigned int, 4u>*, unsigned long)"


def _write(directory, counter, values):
    os.makedirs(directory)
    with open(os.path.join(directory, "p_counter_collection.csv"), "w", newline="") as f:
        w = csv.DictWriter(f, fieldnames=["Kernel_Name", "Counter_Name", "Counter_Value"])
        w.writeheader()
        for kernel, vals in values.items():
            for v in vals:
                w.writerow({"Kernel_Name": kernel, "Counter_Name": counter, "Counter_Value": v})


def test_traffic_picks_the_split_pages_kernel_and_scales_by_the_copy(tmp_path):
    # the copy of 1 MiB reads as 512 KiB fetched (counter counts half) and 1024 KiB written
    _write(str(tmp_path / "fetch"), "FETCH_SIZE", {COPY: [512.0, 512.0], SPARSE: [100.0, 300.0], MANY_ROWS: [9000.0]})
    _write(str(tmp_path / "write"), "WRITE_SIZE", {COPY: [1024.0], SPARSE: [10.0, 30.0], MANY_ROWS: [7000.0]})
    r = subprocess.run([sys.executable, "-m", "paper_2604_12056_amd.profile_summary", "traffic", str(tmp_path / "fetch"),
                        str(tmp_path / "write"), "--copy-bytes", str(1 << 20)], capture_output=True, text=True, cwd=ROOT)
    assert r.returncode == 0, r.stderr
    vals = dict(line.split(": ") for line in r.stdout.splitlines() if line.startswith("attn_"))
    # mean 200 KiB fetched x 1024 x scale 2.0; mean 20 KiB written x 1024 x scale 1.0: the many-row
    # kernel, whose name also carries a "true", is not the one reported
    assert float(vals["attn_fetch_bytes_per_launch"]) == 200.0 * 1024 * 2.0
    assert float(vals["attn_write_bytes_per_launch"]) == 20.0 * 1024 * 1.0


def test_counters_reports_means_and_busy_fractions(tmp_path):
    """A kernel that keeps all 256 compute units busy for 1000 cycles, its matrix cores for 400 of
    them on every one of the 1024 SIMDs and its vector ALUs for 150 four-cycle issue slots."""
    d = str(tmp_path / "run")
    os.makedirs(d)
    with open(os.path.join(d, "p_counter_collection.csv"), "w", newline="") as f:
        w = csv.DictWriter(f, fieldnames=["Kernel_Name", "Counter_Name", "Counter_Value"])
        w.writeheader()
        for name, vals in (("SQ_BUSY_CU_CYCLES", [256e3, 256e3]), ("SQ_VALU_MFMA_BUSY_CYCLES", [400.0 * 1024] * 2),
                           ("SQ_ACTIVE_INST_VALU", [150.0 * 1024, 150.0 * 1024])):
            for v in vals:
                w.writerow({"Kernel_Name": MANY_ROWS, "Counter_Name": name, "Counter_Value": v})
    r = subprocess.run([sys.executable, "-m", "paper_2604_12056_amd.profile_summary", "counters", d], capture_output=True,
                       text=True, cwd=ROOT)
    assert r.returncode == 0, r.stderr
    lines = {" ".join(l.split()[:-1]): l.split()[-1] for l in r.stdout.splitlines() if l.startswith("    ")}
    assert float(lines["matrix-core busy / duration"]) == 0.4
    assert float(lines["vector-ALU issue busy / duration"]) == 0.6
    assert "launches 2" in r.stdout
