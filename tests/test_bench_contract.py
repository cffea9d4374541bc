"""bench.py's control flow and the shape of its one JSON line, without a GPU: the device pieces (events,
synchronisation, the decode call, the MFMA probe) are replaced by stand-ins, everything else is the real
script -- argument handling, the choice among the variants, the side-by-side leg, the oracle timed as the
CPU baseline.  No kernel runs and no figure in the output means anything; the keys and their types do."""
import io
import json
import os
import sys
import time
from contextlib import redirect_stdout

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


class _Event:
    def __init__(self, enable_timing=False):
        self.t = None

    def record(self):
        self.t = time.perf_counter()

    def elapsed_time(self, other):
        return (other.t - self.t) * 1e3 + 1e-3


@pytest.fixture
def fake_gpu(monkeypatch):
    import torch
    sys.path.insert(0, ROOT)
    amla = pytest.importorskip("paper_2509_25224_amd.amla")
    cpu = torch.device("cpu")
    monkeypatch.setattr(torch.cuda, "is_available", lambda: True)
    monkeypatch.setattr(torch.cuda, "synchronize", lambda *a, **k: None)
    monkeypatch.setattr(torch.cuda, "Event", _Event)
    monkeypatch.setattr(torch, "device", lambda *a, **k: cpu)
    calls = []

    def decode(q, kv, tab, lens, scale, out=None, lse=None, *, variant=1, num_splits=0, flags=0, workspace=None,
               want_lse=True, q_lens=None):
        calls.append((variant, flags))
        out.fill_(0.5)
        lse.fill_(1.0)
        return out, lse

    monkeypatch.setattr(amla, "amla_decode", decode)
    monkeypatch.setattr(amla, "amla_mfma_probe", lambda iters, wgs: 1e12)
    return calls


def _run(monkeypatch, argv):
    import bench
    monkeypatch.setattr(sys, "argv", ["bench.py"] + argv)
    buf = io.StringIO()
    with redirect_stdout(buf):
        bench.main()
    lines = [ln for ln in buf.getvalue().splitlines() if ln.strip()]
    assert len(lines) == 1                                   # exactly one JSON line
    return json.loads(lines[0])


def test_default_line_has_the_contract_keys(fake_gpu, monkeypatch):
    r = _run(monkeypatch, ["--config", "0", "--steps", "3", "--warmup", "1"])
    for key, kind in (("metric", str), ("value", float), ("unit", str), ("n_gpus", int), ("steps", int), ("warmup", int),
                      ("ms_per_step", float), ("higher_is_better", bool), ("scaling", str), ("dtype", str), ("data", str),
                      ("config", dict), ("roofline", dict), ("cpu_baseline", dict)):
        assert isinstance(r[key], kind), key
    assert r["n_gpus"] == 1 and r["steps"] == 3 and r["warmup"] == 1 and r["vs_baseline"] is None
    assert r["unit"] == "TFLOP/s" and r["higher_is_better"] is True and r["data"] == "synthetic" and r["dtype"] == "bf16"
    assert "workload" in r["config"] and "model" not in r["config"]
    roof = r["roofline"]
    assert roof["bound"] == "mfma" and roof["unit"] == "TFLOP/s" and roof["peak"] == pytest.approx(2516.6)
    assert roof["frac"] == pytest.approx(roof["achieved"] / roof["peak"]) and "traffic" in roof
    assert roof["kernel"].startswith("amla_decode")
    cpu = r["cpu_baseline"]
    assert cpu["kind"] == "oracle" and cpu["unit"] == "TFLOP/s" and cpu["cores"] >= 1 and cpu["value"] > 0 and cpu["sample"]
    # the headline kernel is fixed: the strict exponent add on the default (row-rescale) kernels
    assert r["config"]["variant"] == "add" and roof["kernel"] == "amla_decode_rg_kernel"
    assert r["config"]["decomposition"] == "equal_share" and r["config"]["kv_splits"] >= 1
    par = r["parity"]
    assert par["rows_checked"] > 0 and par["kernel"] == roof["kernel"] and par["variant"] == "add"
    assert isinstance(par["max_out_err"], float) and isinstance(par["max_lse_err"], float) and par["passed"] is False
    assert {"mul", "add", "add_comp", "mul_512", "add_512", "mul_t", "add_t", "mul_lazy", "add_lazy", "add_ldexp"} <= set(r["rescale"]["tflops"])
    assert r["rescale"]["add_over_mul_speedup"] > 0 and r["rescale"]["add_t_over_mul_t_speedup"] > 0


def test_a_named_variant_is_the_one_timed(fake_gpu, monkeypatch):
    from paper_2509_25224_amd import amla
    r = _run(monkeypatch, ["--config", "0", "--steps", "2", "--warmup", "0", "--variant", "mul_lazy", "--no-ab",
                           "--no-cpu-baseline", "--no-mfma-probe"])
    assert r["config"]["variant"] == "mul_lazy" and r["roofline"]["kernel"] == "amla_decode_kernel"
    assert set(fake_gpu) == {(amla.AMLA_RESCALE_MUL, amla.AMLA_FLAG_LAZY_RESCALE)}
    assert "cpu_baseline" not in r and "rescale" not in r and "parity" not in r


def test_balanced_decomposition_names_its_kernel(fake_gpu, monkeypatch):
    from paper_2509_25224_amd import amla
    r = _run(monkeypatch, ["--config", "0", "--steps", "2", "--warmup", "0", "--balanced", "--no-ab",
                           "--no-cpu-baseline", "--no-mfma-probe"])
    assert r["roofline"]["kernel"] == "amla_decode_rg_balanced_kernel" and r["config"]["decomposition"] == "balanced"
    assert set(fake_gpu) == {(amla.AMLA_RESCALE_ADD, amla.AMLA_FLAG_BALANCED)}


def test_more_than_one_gpu_is_refused(monkeypatch):
    import bench
    monkeypatch.setattr(sys, "argv", ["bench.py", "--gpus", "2"])
    with pytest.raises(SystemExit) as e:
        bench.main()
    assert e.value.code != 0
