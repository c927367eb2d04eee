"""The committed counter profile covers the kernels bench.py reports rooflines for: `roofline.traffic` is looked up
there by kernel name and configuration, so a kernel that was renamed (a template parameter added) without the
profile being taken again would silently lose its traffic figure."""
import importlib.util
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _bench():
    spec = importlib.util.spec_from_file_location("loma_bench", os.path.join(ROOT, "bench.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)      # defines functions and tables only; main() runs under __main__
    return mod


def test_every_roofline_kernel_has_a_traffic_figure_in_the_committed_profile():
    bench = _bench()
    table = bench.profile_traffic()
    assert table, "profiles/bench_hbm_traffic_pmc.md is missing or has no calibration table"
    for which, (config, kernels) in bench.ROOFLINE_KERNELS.items():
        if "{L}" in config:
            continue      # the layered decode is profiled with two layer caches per launch; the default run uses 32
        got = bench.traffic_of(table, config, *kernels)
        assert got is not None and got > 0, f"{which}: {kernels} @{config} not in the counter profile"


def test_traffic_figures_are_at_least_the_algorithmic_bytes():
    """Counter traffic below the tensors' own bytes would mean a wrong calibration factor or a wrong row."""
    text = open(os.path.join(ROOT, "profiles", "bench_hbm_traffic_pmc.md")).read()
    rows = re.findall(r"^\|\s*`([^`]+)`\s*\|([^|]*)\|\s*\d+\s*\|[^|]*\|[^|]*\|\s*([0-9.]+)\s*\|\s*([0-9.]+)\s*\|\s*([0-9.]+)\s*\|", text, flags=re.M)
    assert len(rows) >= 6
    for kernel, workload, traffic, algorithmic, ratio in rows:
        if float(algorithmic) == 0:
            continue
        assert 0.98 <= float(traffic) / float(algorithmic) < 3.0, (kernel, workload, traffic, algorithmic)
        assert abs(float(traffic) / float(algorithmic) - float(ratio)) < 0.02


def test_profiled_kernels_are_the_ones_the_sources_define():
    """Every kernel named in the profile is a template the HIP sources define, with as many arguments."""
    bench = _bench()
    src = "".join(open(os.path.join(ROOT, "paper_2401_09486_amd", "csrc", f)).read()
                  for f in os.listdir(os.path.join(ROOT, "paper_2401_09486_amd", "csrc")) if f.endswith((".hip", ".h")))
    for which, (_, kernels) in bench.ROOFLINE_KERNELS.items():
        for k in kernels:
            name, args = re.match(r"(\w+)<(.*)>$", k).groups()
            m = re.search(r"template\s*<([^>]*)>\s*__global__[^;{]*?\bvoid\s+" + name + r"\s*\(", src, flags=re.S)
            assert m, f"{which}: no kernel template named {name}"
            assert len(m.group(1).split(",")) == len(args.split(",")), f"{which}: {k} does not match template <{m.group(1)}>"
