"""CPU-only checks of the measurement records bench.py reads: every HBM-traffic summary under profiles/ names the
kernel sources it was measured on and carries a traffic figure that can belong to the workload it is for."""
import glob
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _field(text, name):
    m = re.search(r"^%s:\s*(.+)$" % re.escape(name), text, re.M)
    return None if m is None else m.group(1).strip()


def test_traffic_summaries_are_plausible_and_stamped():
    files = sorted(glob.glob(os.path.join(ROOT, "profiles", "*_hbm_traffic.txt")))
    assert len(files) >= 8
    for path in files:
        text = open(path).read()
        alg = float(_field(text, "algorithmic_bytes_per_launch"))
        traffic = float(_field(text, "traffic_bytes_per_launch"))
        ratio = float(_field(text, "traffic_over_algorithmic"))
        # a kernel cannot move fewer bytes than the method needs, and none of these re-reads its cache: the measured
        # ratios are 1.0001 (plain decode) to 1.03 (the forms that stage scores); a figure far outside says that the
        # counters were scaled wrongly, not that the kernel changed
        assert abs(traffic / alg - ratio) < 1e-3, path
        assert 0.99 <= ratio <= 1.10, (path, ratio)
        # the calibration copy moves 4 GiB each way: FETCH_SIZE counts it in units of 2 KiB, WRITE_SIZE in KiB
        scales = [float(x) for x in re.findall(r"-> scale x([0-9.]+)", text)]
        assert len(scales) == 2 and abs(scales[0] - 2.0) < 0.01 and abs(scales[1] - 1.0) < 0.01, (path, scales)
        srcs = _field(text, "kernel_sources").split()
        assert srcs and re.fullmatch(r"[0-9a-f]{16}", _field(text, "kernel_sources_sha16")), path
        for name in srcs:
            assert os.path.exists(os.path.join(ROOT, "paper_2408_05646_amd", "csrc", name)) or \
                os.path.exists(os.path.join(ROOT, "include", name)), (path, name)
        assert "rocprofv3 --pmc FETCH_SIZE" in text and "rocprofv3 --pmc WRITE_SIZE" in text, path


def test_every_profile_summary_names_its_command_and_its_kernel_sources():
    """Every summary under profiles/ is text, gives the rocprofv3 command that made it (which runs committed files
    only), names the kernel sources it was measured on -- files that exist -- and carries their hash."""
    files = sorted(glob.glob(os.path.join(ROOT, "profiles", "*")))
    assert len(files) >= 20
    for path in files:
        assert path.endswith((".txt", ".md")), path
        text = open(path).read()
        assert len(text) < 40000, path                                  # a summary, not raw profiler output
        assert "rocprofv3" in text and "bench.py" in text and "_work" not in text, path
        srcs = _field(text, "kernel_sources").split()
        assert srcs and re.fullmatch(r"[0-9a-f]{16}", _field(text, "kernel_sources_sha16")), path
        for name in srcs:
            assert os.path.exists(os.path.join(ROOT, "paper_2408_05646_amd", "csrc", name)) or \
                os.path.exists(os.path.join(ROOT, "include", name)), (path, name)
