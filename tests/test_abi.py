"""CPU-side checks of the boundary: the library loads and exports every symbol the header declares,
and the Python structs have the C layout.  No compute call is made here."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "psd.h")


def _declared():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    names = set(re.findall(r"\b(psd_[a-z_0-9]+)\s*\(", src))
    names -= {"psd_trace_fn"}
    return sorted(names)


def test_header_declares_the_boundary_calls():
    names = _declared()
    for must in ("psd_create", "psd_generate", "psd_accept", "psd_forward", "psd_destroy", "psd_strerror"):
        assert must in names


def test_library_exports_every_declared_symbol():
    from paper_2510_12966_amd import binding

    path = binding.lib_path()
    if not os.path.exists(path):
        from paper_2510_12966_amd import build
        build.build()
    try:
        lib = ctypes.CDLL(path)
    except OSError as e:
        pytest.skip(f"HIP runtime not loadable here: {e}")
    for name in _declared():
        assert hasattr(lib, name), name
    lib.psd_strerror.restype = ctypes.c_char_p
    assert lib.psd_strerror(0) == b"ok"
    assert b"invalid" in lib.psd_strerror(-1)


def test_struct_layouts_match_the_header():
    from paper_2510_12966_amd import binding as b

    assert ctypes.sizeof(b._ModelDesc) == 6 * 4 + 2 * 4 + 2 * 4 + 8 + 8
    assert b._ModelDesc.weights.offset == 40 and b._ModelDesc.weights_bytes.offset == 48
    assert ctypes.sizeof(b._Params) == 8 * 4 + 8 and b._Params.pool_bytes.offset == 32
    assert ctypes.sizeof(b.Stats) == 9 * 8 + 6 * 8
    assert ctypes.sizeof(b.KernelStat) == 48 + 8 + 8 + 8


def test_binding_has_no_fallback_and_does_not_import_the_oracle():
    import paper_2510_12966_amd.binding as b

    src = open(b.__file__).read() + open(os.path.join(os.path.dirname(b.__file__), "__init__.py")).read()
    assert "oracle" not in src
    assert "is missing" in src   # a missing library is an error, never a silent CPU path


def test_throughput_model_of_section_3_3():
    import bench
    # one stage: beta (l + 1) / (l / V_D + 1 / V_Q); hand-computed: 0.8 * 5 / (4 / 1000 + 1 / 400) = 615.38...
    f_qd, v_psd, v_sd = bench.throughput_model(0.8, 0.9, 4, 8, 1000.0, 400.0, 250.0)
    assert abs(f_qd - 0.8 * 5 / (4 / 1000 + 1 / 400)) < 1e-9 and abs(f_qd - 615.3846153846) < 1e-6
    assert abs(v_psd - 0.9 * 9 / (8 / f_qd + 1 / 250)) < 1e-9
    assert abs(v_sd - 0.9 * 9 / (8 / 400 + 1 / 250)) < 1e-9 and abs(v_sd - 337.5) < 1e-9
    # a faster first stage can only help, and beta = 1, l -> large approaches the proposer's speed
    assert bench.throughput_model(1.0, 1.0, 4, 8, 2000.0, 400.0, 250.0)[1] > v_psd
    assert abs(bench.throughput_model(1.0, 1.0, 10 ** 6, 8, 1000.0, 400.0, 250.0)[0] - 1000.0) < 1.0


def test_bench_reads_measured_traffic_from_the_committed_profile():
    import bench
    val, src = bench.measured_traffic("paper", "gemm_gate_up draft")
    assert src == bench.TRAFFIC_PROFILE and os.path.exists(os.path.join(ROOT, src))
    assert 67.1e6 <= val <= 70e6          # HBM bytes per launch of the dominant kernel: its 67.11 MB of weights plus ~1 %
    assert bench.measured_traffic("paper", "no such kernel") == (None, None)


def test_adaptive_structs_have_the_same_layout_on_both_sides():
    import oracle
    from paper_2510_12966_amd import binding as b
    assert ctypes.sizeof(b.Adapt) == ctypes.sizeof(oracle.Adapt) == 5 * 4 + 4 * 4
    assert [n for n, _ in b.Adapt._fields_] == [n for n, _ in oracle.Adapt._fields_]


def test_bench_cost_model_arithmetic():
    import bench
    rows = [{"name": "gemm_gate_up draft w<=1", "launches": 160, "bytes_total": 160 * 67.1e6},
            {"name": "gemm_gate_up draft w<=512", "launches": 16, "bytes_total": 16 * 67.1e6},   # ingestion: left out
            {"name": "sample draft", "launches": 10, "bytes_total": 10 * 513e3},                  # two launches per unit
            {"name": "attn target w<=12", "launches": 32, "bytes_total": 32 * 1e6}]
    cm = bench.cost_model(rows, {"draft": 10, "qualifier": 0, "target": 1}, {"draft": 0.3, "qualifier": 0.0, "target": 0.2})
    d = cm["pass"]["draft"]
    assert d["launches"] == 18.0 and abs(d["GB"] - 1.074) < 1e-3
    # 18 launches x 4.3 us + 1.0741 GB at 6.6 TB/s = 0.0774 + 0.1627 ms
    assert abs(d["predicted_ms"] - (18 * 4.3e-3 + 1.0741e9 / 6.6e9)) < 1e-3 and abs(d["measured_over_predicted"] - 0.3 / 0.2401) < 2e-3
    assert "qualifier" not in cm["pass"] and cm["pass"]["target"]["launches"] == 32.0
