"""Host-side checks that need no GPU: the shared library loads and exports every symbol that
include/dz.h declares; size formula; oracle and product do not import each other."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "dz.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dz_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    import paper_2312_05215_amd as dz
    L = dz.lib()
    names = _declared()
    assert len(names) >= 12
    for n in names:
        assert hasattr(L, n), n
    assert sorted(dz.SYMBOLS) == names


def test_packed_bytes_closed_form():
    import paper_2312_05215_amd as dz
    # bits per dense weight: (2b+4)/4 for codes+positions, 32/G for scale+zero
    assert dz.dz_packed_bytes(4096, 4096, 4, 128) * 8 == int(4096 * 4096 * 3.25)
    assert dz.dz_packed_bytes(4096, 4096, 2, 128) * 8 == int(4096 * 4096 * 2.25)
    assert dz.dz_packed_bytes(256, 256, 4, 64) * 8 == int(256 * 256 * 3.5)
    for N, K, b, G in [(11008, 4096, 4, 128), (4096, 11008, 2, 128), (28672, 8192, 2, 128), (1024, 8192, 2, 64)]:
        assert dz.dz_packed_bytes(N, K, b, G) == N * K * (2 * b + 4) // 32 + 4 * N * K // G
    assert dz.dz_strerror(0) == "ok"


def test_oracle_and_product_are_independent():
    def imports(path):
        out = []
        for dirpath, _, files in os.walk(path):
            for f in files:
                if f.endswith((".py", ".c", ".h", ".hip", ".cpp")):
                    out.append(open(os.path.join(dirpath, f)).read())
        return "\n".join(out)
    prod = imports(os.path.join(ROOT, "paper_2312_05215_amd"))
    orc = imports(os.path.join(ROOT, "oracle"))
    assert "oracle" not in prod
    assert "paper_2312_05215_amd" not in orc and "libdz.so" not in orc and "csrc" not in orc


def test_committed_traffic_summaries_are_readable_by_the_benchmark():
    """bench.py fills roofline.traffic from profiles/<kernel>_<workload>_pmc.txt; every performance workload
    has one, and the figure is at least the algorithmic bytes' order of magnitude."""
    import importlib.util
    import os
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    spec = importlib.util.spec_from_file_location("bench_module", os.path.join(root, "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    for kernel, workload, launches in (("stream_kernel", "7b_decode", 4), ("stream_kernel", "7b_decode_many", 4),
                                       ("stream_kernel", "70b_stack", 4), ("prefill_kernel", "13b_prefill", 7)):
        traffic, src = bench.profile_traffic(kernel, workload, launches)
        assert traffic is not None and traffic > 100e6, (kernel, workload, traffic)
        assert src == os.path.join("profiles", f"{kernel}_{workload}_pmc.txt")
        assert bench.profile_traffic(kernel, workload, launches + 1) == (None, None)      # other launch grouping: no figure
