"""The rocprofv3 summaries under profiles/ that bench.py reads at run time: the traffic table parses and
covers the GEMM shapes of the default line and of the spec block."""
import importlib.util
import os

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _bench():
    spec = importlib.util.spec_from_file_location("bench_module", os.path.join(ROOT, "bench.py"))
    m = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(m)
    return m


def test_traffic_table_covers_the_benchmarked_shapes():
    bench = _bench()
    from paper_2311_01305_amd import synth
    table = bench.measured_gemm_traffic()
    for cfg in (bench.DEFAULT_CFG, 3):
        wl = synth.WORKLOADS[cfg]
        for lin in wl.linears:
            f, w, name = table[(wl.T, lin.N, lin.K)]
            algorithmic = (wl.T * lin.K + lin.N * lin.K + 4 * wl.T * lin.N) / 1e9
            # the output is written once; the fills exceed the operands (per-XCD L2s) but stay bounded
            assert 0.95 * 4 * wl.T * lin.N / 1e9 <= w <= 1.15 * 4 * wl.T * lin.N / 1e9, (cfg, lin.name)
            assert f + w >= algorithmic and f < 60 * (wl.T * lin.K + lin.N * lin.K) / 1e9 and name.endswith(".txt")
    roof = bench.gemm_roofline([(l.N, l.K) for l in synth.WORKLOADS[bench.DEFAULT_CFG].linears], synth.T_FULL, 7 * 20.0, 7)
    assert roof["unit"] == "TOP/s" and roof["bound"] == "mfma" and roof["traffic"] is not None
    assert abs(roof["frac"] - roof["achieved"] / 5000.0) < 1e-12


def test_profile_summaries_name_their_commands():
    names = [f for f in os.listdir(os.path.join(ROOT, "profiles")) if f.endswith(".txt")]
    assert names
    for f in names:
        text = open(os.path.join(ROOT, "profiles", f)).read()
        assert "bench.py" in text and ("rocprofv3" in text or "python3 bench.py" in text), f
