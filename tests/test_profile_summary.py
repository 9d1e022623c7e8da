"""The rocprofv3 summary script on made-up counter tables: the HBM bytes of a call are scaled by
what the same counter reads for the 1 GiB calibration copy, and a call that splits into several
launches is charged the sum of its launches."""
import subprocess
import sys
from pathlib import Path

ROOT = Path(__file__).resolve().parents[1]
COPY = "(anonymous namespace)::copy_kernel(HIP_vector_type<unsigned int, 4u>*, HIP_vector_type<unsigned int, 4u> const*, unsigned long)"
WAVE = "void (anonymous namespace)::emb_bag_wave_kernel<16, 0, 4, 0, true>(char const*, long const*)"
STREAM = "void (anonymous namespace)::emb_bag_stream_kernel<16, 0, 4, false, false>(char const*, long const*)"
OTHER = "void at::native::vectorized_elementwise_kernel<16, at::native::FillFunctor<unsigned char> >(int)"


def _counter_csv(path, counter, rows):
    lines = ['"Dispatch_Id","Kernel_Name","Counter_Name","Counter_Value"']
    for i, (kernel, value) in enumerate(rows):
        lines.append(f'{i},"{kernel}","{counter}",{value}')
    path.write_text("\n".join(lines) + "\n")
    return str(path)


def _run(*args):
    r = subprocess.run([sys.executable, "-m", "paper_2410_22249_amd.profile_summary", *args],
                       cwd=ROOT, capture_output=True, text=True, check=True)
    return dict(l.split(" = ")[0:2] for l in r.stdout.splitlines() if " = " in l), r.stdout


def test_one_launch_per_call_is_scaled_by_the_calibration_copy(tmp_path):
    # the copy of 1 GiB reads as half of it: every fetched KiB counts twice
    fetch = _counter_csv(tmp_path / "f.csv", "FETCH_SIZE",
                         [(COPY, 524288.0), (OTHER, 7.0)] + [(WAVE, v) for v in (1000.0, 1002.0, 5000.0)])
    write = _counter_csv(tmp_path / "w.csv", "WRITE_SIZE",
                         [(COPY, 1048576.0)] + [(WAVE, v) for v in (300.0, 300.0, 300.0)])
    got, text = _run("--workload", "x", "--fetch", fetch, "--write", write)
    assert float(got["fetch_bytes_per_launch"]) == 1002.0 * 1024 * 2       # the median, scaled by 2
    assert float(got["write_bytes_per_launch"]) == 300.0 * 1024
    assert float(got["hbm_bytes_per_launch"].split()[0]) == 1002.0 * 2048 + 300.0 * 1024


def test_a_split_call_is_charged_the_sum_of_its_launches(tmp_path):
    rows = [(COPY, 1048576.0)]
    for _ in range(4):                       # each call: one stream launch, then one wave launch
        rows += [(STREAM, 100.0), (WAVE, 4000.0)]
    fetch = _counter_csv(tmp_path / "f.csv", "FETCH_SIZE", rows)
    write = _counter_csv(tmp_path / "w.csv", "WRITE_SIZE", rows)
    occ = _counter_csv(tmp_path / "o.csv", "MeanOccupancyPerCU",
                       [(STREAM, 20.0), (WAVE, 28.0), (STREAM, 22.0), (WAVE, 30.0)])
    got, text = _run("--workload", "x", "--fetch", fetch, "--write", write, "--counters", occ)
    assert float(got["fetch_bytes_per_call"]) == 4100.0 * 1024
    assert float(got["hbm_bytes_per_launch"].split()[0]) == 2 * 4100.0 * 1024
    assert "one call = 2 launches" in text
    occ_lines = [l for l in text.splitlines() if l.startswith("MeanOccupancyPerCU")]
    assert len(occ_lines) == 2 and "21.000" in occ_lines[0] and "29.000" in occ_lines[1]


def test_missing_calibration_copy_is_reported_not_guessed(tmp_path):
    fetch = _counter_csv(tmp_path / "f.csv", "FETCH_SIZE", [(WAVE, 1000.0)])
    got, text = _run("--workload", "x", "--fetch", fetch)
    assert not got and "calibration copy or embedding kernel not found" in text
