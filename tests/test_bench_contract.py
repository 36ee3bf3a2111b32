"""Static checks of bench.py that need no GPU: the one-GPU rule, and that every stored traffic figure names a
summary under profiles/ that exists and quotes the kernel variant it was measured on."""
import os
import re
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _bench_source():
    with open(os.path.join(ROOT, "bench.py")) as f:
        return f.read()


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=300)
    assert r.returncode != 0
    assert "one GPU" in r.stderr
    assert not r.stdout.strip()  # no JSON line


def test_stored_traffic_figures_point_at_existing_summaries_of_the_same_kernel():
    src = _bench_source()
    table = src[src.index("MEASURED_TRAFFIC = ["):]
    table = table[: table.index("]\n") + 1]
    ns = {}
    exec(table, ns)  # a literal list of dicts
    entries = ns["MEASURED_TRAFFIC"]
    assert entries
    for e in entries:
        path = os.path.join(ROOT, e["source"])
        assert os.path.isfile(path), e["source"]
        text = open(path).read()
        # the summary lists the kernel whose template arguments the variant string abbreviates
        kernel = e["variant"].split("<")[0]
        assert kernel in text, (kernel, e["source"])
        # ... and its scaled bytes beyond L2, to three digits
        gb = f"{e['bytes_beyond_l2'] / 1e9:.3f} GB"
        assert gb in text, (gb, e["source"])
        assert re.match(r"k_[a-z_]+<[-0-9a-z,]+> groups/block=\d+ ngs=\d+ waves/block=\d+ flush=(ordered|atomic) tiles=", e["variant"])


def test_the_json_line_carries_the_required_objects():
    src = _bench_source()
    for key in ('"metric"', '"value"', '"unit"', '"n_gpus"', '"steps"', '"warmup"', '"ms_per_step"', '"higher_is_better"',
                '"scaling"', '"vs_baseline"', '"dtype"', '"data"', '"config"', '"roofline"', '"cpu_baseline"', '"bound"',
                '"achieved"', '"peak"', '"frac"', '"traffic"'):
        assert key in src, key


def test_every_command_quoted_in_profiles_uses_options_that_bench_defines():
    src = _bench_source()
    defined = set(re.findall(r'add_argument\("(--[a-z0-9-]+)"', src))
    assert "--config" in defined and "--steps" in defined
    prof = os.path.join(ROOT, "profiles")
    seen = 0
    for name in sorted(os.listdir(prof)):
        assert name.endswith((".md", ".txt")), name  # summaries only, nothing that runs
        text = open(os.path.join(prof, name)).read()
        assert "rocprofv3" in text, name  # each summary gives the command that made it
        for line in text.splitlines():
            if "bench.py" not in line or "rocprofv3" not in line:
                continue
            args = line.split("bench.py", 1)[1]
            for opt in re.findall(r"(--[a-z0-9-]+)", args):
                assert opt in defined, (name, opt)
                seen += 1
    assert seen > 20
