"""The two measurement aids the design notes quote ceilings from, run on the GPU.

tests/native/probe_gather.hip: the multiply phase's access pattern alone (random 128-byte rows of an
L2-resident panel); tests/native/probe_mfma.hip: back-to-back fp32 matrix instructions.  The test
prints what they measure and only checks that the figures are sane (the notes quote the values of a
run, `profiles/probes_gather_mfma.md`); the libraries are built by __graft_entry__.build().
"""
import ctypes as C
import os

import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

HERE = os.path.join(os.path.dirname(os.path.abspath(__file__)), "native")


def run(lib_name, fn_name):
    path = os.path.join(HERE, lib_name)
    assert os.path.exists(path), f"{path} is missing: run __graft_entry__.build()"
    assert torch.cuda.is_available(), "GPU tests need a device"
    fn = getattr(C.CDLL(path), fn_name)
    fn.argtypes = [C.POINTER(C.c_double), C.c_int]
    fn.restype = C.c_int
    rates = (C.c_double * 16)()
    print(f"[case] {fn_name}", flush=True)
    count = fn(rates, 16)
    assert count > 0, f"{fn_name} failed: {count}"
    return [rates[i] for i in range(count)]


def test_gather_probe_reports_a_rate_below_the_l1_fill_peak():
    rates = run("libprobe_gather.so", "probe_gather")
    print("gather probe, TB/s:", [round(r, 1) for r in rates], flush=True)
    # 256 CUs x 64 B per clock at 2.4 GHz = 39.3 TB/s is what the L1s can take at most
    assert 5.0 < max(rates) < 39.4


def test_mfma_probe_reports_a_rate_below_the_fp32_peak():
    rates = run("libprobe_mfma.so", "probe_mfma")
    print("matrix-core probe, TFLOP/s:", [round(r, 1) for r in rates], flush=True)
    assert 50.0 < max(rates) < 157.4
