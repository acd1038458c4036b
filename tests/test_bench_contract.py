"""Host-side checks of bench.py that need no GPU: every option the code reads is one the parser defines,
more than one GPU is refused, and the stored counter figures belong to the kernel sources in the tree."""
import ast
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
BENCH = os.path.join(ROOT, "bench.py")


def test_every_option_read_is_defined():
    tree = ast.parse(open(BENCH).read())
    read = {n.attr for n in ast.walk(tree)
            if isinstance(n, ast.Attribute) and isinstance(n.value, ast.Name) and n.value.id == "args"}
    defined = set()
    for n in ast.walk(tree):
        if isinstance(n, ast.Call) and isinstance(n.func, ast.Attribute) and n.func.attr == "add_argument":
            flag = n.args[0].value
            assert flag.startswith("--")
            defined.add(flag[2:].replace("-", "_"))
    assert read <= defined, sorted(read - defined)


def test_more_than_one_gpu_is_refused():
    r = subprocess.run([sys.executable, BENCH, "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "--gpus 1" in r.stderr


def test_stored_traffic_names_known_workloads():
    sys.path.insert(0, ROOT)
    import bench
    from paper_2512_21450_amd import workloads as wl
    for name, t in bench.PMC_TRAFFIC.items():
        if name == "csrc_sha256":
            assert t == "" or len(t) == 64
            continue
        assert name in wl.WORKLOADS
        assert t["fetch_bytes"] >= 0 and t["write_bytes"] >= 0
    # the hash covers the files the K/V-streaming kernel is built from
    assert len(bench.csrc_sha256()) == 64


def test_source_hash_ignores_comments_and_layout_only():
    sys.path.insert(0, ROOT)
    import bench
    a = 'int f(int x) { // doubles\n  return 2 * x; /* twice */ }\nconst char* s = "// kept";\n'
    b = 'int f(int x) {\n\n  return 2 * x;  }   const char* s = "// kept";'
    c = 'int f(int x) { return 3 * x; } const char* s = "// kept";'
    assert bench.strip_comments(a) == bench.strip_comments(b) != bench.strip_comments(c)
    assert '"// kept"' in bench.strip_comments(a)
