"""Control flow of the Algorithm 1 step controller, checked on the CPU with the C-ABI calls replaced by
recorders (no kernel runs here; the GPU parity tests run the real thing)."""
import pytest
import torch

from paper_2509_24014_amd import binding, schedule


@pytest.fixture
def recorder(monkeypatch):
    log = []
    monkeypatch.setattr(binding, "attn_dense", lambda q, k, v, out=None, lse_out=None, stream=None:
                        log.append(("dense", lse_out is not None)) or q)
    monkeypatch.setattr(binding, "attn_sparse", lambda q, k, v, index, out=None, stream=None:
                        log.append(("sparse", index)) or q)
    monkeypatch.setattr(binding, "select_workspace_bytes", lambda q, bq, bk: 16)

    def fake_select(q, k, bq, bk, rho, lse_in=None, workspace=None, pooled_out=None, index=None, stream=None):
        log.append(("select", lse_in is not None))
        return ("index", sum(1 for e in log if e[0] == "select"))

    monkeypatch.setattr(binding, "select_pattern", fake_select)
    return log


def _run(layer, T):
    q = torch.zeros(1, 1, 64, 64)
    for t in range(T):
        layer.step(q, q, q, t)


def test_default_schedule_selects_once_at_the_last_dense_step(recorder):
    layer = schedule.SparseDLayer(10, 0.3, 32, 32, 0.5)
    assert layer.n_dense == 3
    _run(layer, 10)
    kinds = [e[0] for e in recorder]
    assert kinds == ["dense", "dense", "dense", "select"] + ["sparse"] * 7
    assert recorder[0] == ("dense", False) and recorder[2] == ("dense", True)   # only the switch step emits the log-sum-exp
    assert recorder[3] == ("select", True)                                       # and selection reuses it
    assert all(e[1] == ("index", 1) for e in recorder if e[0] == "sparse")       # one pattern, reused unchanged
    assert layer.calls == {"dense": 3, "select": 1, "sparse": 7}


def test_without_skipping_selects_at_step_zero(recorder):
    layer = schedule.SparseDLayer(4, 0.0, 32, 32, 0.5, n_dense=0)
    _run(layer, 4)
    assert [e[0] for e in recorder] == ["select", "sparse", "sparse", "sparse", "sparse"]
    assert recorder[0] == ("select", False)   # no dense call to take statistics from
    assert layer.calls == {"dense": 0, "select": 1, "sparse": 4}


def test_without_reuse_reselects_every_sparse_step(recorder):
    layer = schedule.SparseDLayer(5, 0.4, 32, 32, 0.5, reselect_every_step=True)
    _run(layer, 5)
    assert [e[0] for e in recorder] == ["dense", "dense", "select", "select", "sparse", "select", "sparse", "select", "sparse"]
    assert layer.calls == {"dense": 2, "select": 4, "sparse": 3}


def test_sparse_step_before_selection_is_an_error(recorder):
    layer = schedule.SparseDLayer(5, 0.4, 32, 32, 0.5)
    q = torch.zeros(1, 1, 64, 64)
    with pytest.raises(RuntimeError):
        layer.step(q, q, q, 3)


def test_bench_refuses_more_than_one_gpu():
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "ONE GPU" in r.stderr and r.stdout.strip() == ""
