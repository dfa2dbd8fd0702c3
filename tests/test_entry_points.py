"""The command-line and import contracts that need no GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_refuses_more_than_one_gpu():
    """This build runs on one GPU: bench.py --gpus 2 exits with a message instead of measuring."""
    proc = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                          stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, cwd=ROOT, timeout=120)
    assert proc.returncode == 2
    assert "one GPU" in proc.stderr and proc.stdout.strip() == ""


def test_binding_fails_loudly_without_the_built_library():
    """No fallback path: with the library missing, importing the binding raises."""
    code = "import paper_2602_12151_amd.binding"
    env = dict(os.environ, OSERVE_LIB=os.path.join(ROOT, "does_not_exist", "liboserve.so"))
    proc = subprocess.run([sys.executable, "-c", code], stdout=subprocess.PIPE, stderr=subprocess.PIPE,
                          text=True, cwd=ROOT, env=env, timeout=120)
    assert proc.returncode != 0
    assert "ImportError" in proc.stderr and "no fallback" in proc.stderr


def test_product_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2602_12151_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".cpp", ".hip", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower() or f == "workloads.py" and "oracle" in text.lower(), f


def test_bench_settling_phase_terminates_and_reports():
    """The untimed settling phase of bench.py stops after its patience or its cap, whatever the step does."""
    import importlib, time, types
    bench = importlib.import_module("bench")
    fake_torch = types.SimpleNamespace(cuda=types.SimpleNamespace(synchronize=lambda: None))
    calls = []
    assert bench.settle(lambda i: calls.append(i), fake_torch, 0) == (0.0, 0) and not calls
    t0 = time.perf_counter()
    seconds, steps = bench.settle(lambda i: time.sleep(0.002), fake_torch, 0.5)
    assert 0.5 <= seconds < 2.0 and steps > 10 and time.perf_counter() - t0 < 3.0


def test_recorded_traffic_belongs_to_the_current_sources():
    """bench.py reports the split kernel's recorded HBM traffic only while the decode sources are the ones it was
    measured on; this fails when they change, until the profile is taken again and the record renewed."""
    import importlib
    bench = importlib.import_module("bench")
    rec = bench.RECORDED_TRAFFIC
    assert rec["sources_sha16"] == bench.sources_sha16(), (
        "decode sources changed since " + rec["profile"] + " was taken: profile again and renew RECORDED_TRAFFIC")
    assert os.path.exists(os.path.join(ROOT, rec["profile"]))
    # traffic cannot be below the algorithmic bytes of the workload it was measured on, nor far above
    from paper_2602_12151_amd import workloads as wl
    w = wl.WORKLOADS[rec["config"]]
    algorithmic = wl.kv_bytes(wl.context_lens(w), w.num_kv_heads, w.head_dim)
    assert algorithmic <= rec["bytes"] <= 1.05 * algorithmic


def test_header_is_plain_c():
    """include/oserve.h is a C header: it compiles as C99 without warnings, and a C program can name every
    entry point it declares (link-time check against the built library)."""
    import re, tempfile
    header = open(os.path.join(ROOT, "include", "oserve.h")).read()
    names = sorted(set(re.findall(r"\b(oserve_[a-z0-9_]+)\s*\(", header)))
    assert len(names) > 40
    body = "".join(f"    sink += (unsigned long)(void*)&{n};\n" for n in names)
    src = '#include "oserve.h"\nint main(void) {\n    unsigned long sink = 0;\n' + body + "    return sink == 1;\n}\n"
    with tempfile.TemporaryDirectory() as d:
        c = os.path.join(d, "use_header.c")
        open(c, "w").write(src)
        lib_dir = os.path.join(ROOT, "paper_2602_12151_amd")
        proc = subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror",
                               "-I" + os.path.join(ROOT, "include"), c, "-o", os.path.join(d, "use_header"),
                               "-L" + lib_dir, "-l:liboserve.so", "-Wl,--unresolved-symbols=ignore-in-shared-libs"],
                              stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=120)
        assert proc.returncode == 0, proc.stdout
