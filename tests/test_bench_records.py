"""bench.py prints, beside the figures it measures, a few RECORDED ones read from the rocprofv3
summaries under profiles/.  These checks keep the two from drifting apart silently: every kernel
name bench.py looks up must be a row of the summaries, must be a kernel template that still exists
in the sources with that many template arguments, and the summaries must say which commit they
were taken at."""
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_recorded_figures_resolve_for_every_mapped_pass():
    import bench
    step = {p[1] for p in bench.step_passes()}
    extra = {p[2] for p in bench.extra_passes()}
    for name, kern in bench.KERNEL_OF_PASS.items():
        assert name in step | extra, name
        r = bench.recorded(name)
        assert r["commit"] and re.fullmatch(r"[0-9a-f]{7,40}", r["commit"]), (name, r)
        assert r["traffic"] and r["traffic"] > 1e8, (name, r)
        assert r["valu_per_chunk"] and r["valu_per_chunk"] > 10, (name, r)
        assert r["wait_issue_pct"] is not None and 0 <= r["wait_issue_pct"] <= 100, (name, r)
        assert r["wait_data_pct"] is not None and 0 <= r["wait_data_pct"] <= 100, (name, r)


def test_mapped_kernels_are_instantiations_of_current_templates():
    import bench
    csrc = os.path.join(ROOT, "paper_2605_08565_amd", "csrc")
    text = "".join(open(os.path.join(csrc, f)).read() for f in os.listdir(csrc))
    for kern in set(bench.KERNEL_OF_PASS.values()):
        m = re.fullmatch(r"mxq::(\w+)<(.*)>", kern)
        assert m, kern
        name, args = m.group(1), [a.strip() for a in m.group(2).split(",")]
        decl = re.search(r"template\s*<([^>]*)>\s*__global__\s+void(?:\s+__launch_bounds__\([^)]*\))?\s+" + name + r"\(", text)
        assert decl, f"no kernel template named {name}"
        assert len(decl.group(1).split(",")) == len(args), (kern, decl.group(1))


def test_every_profile_summary_names_its_commit_and_command():
    prof = os.path.join(ROOT, "profiles")
    files = [f for f in os.listdir(prof) if f.endswith((".md", ".txt"))]
    assert len(files) >= 8
    for f in files:
        text = open(os.path.join(prof, f)).read()
        assert re.search(r"Taken at commit `[0-9a-f]{7,40}`", text), f
        assert "bench.py" in text, f
        assert len(text) < 20000, f
