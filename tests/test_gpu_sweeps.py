"""The sweep tool runs end to end on a small shape (every mode prints its table)."""
import sys

import pytest

pytestmark = pytest.mark.gpu


def _run(argv, capsys, monkeypatch):
    from paper_2410_03065_amd import sweeps
    monkeypatch.setattr(sys, "argv", ["sweeps"] + argv)
    sweeps.main()
    return capsys.readouterr().out


def test_sweep_tables_on_a_small_shape(capsys, monkeypatch):
    base = ["--shape", "tiny-f32", "--tokens", "2048", "--budget", "256", "--fetch-unit", "64"]
    out = _run(base + ["--chunks", "--compression", "--lengths", "--gbit", "8", "16"], capsys, monkeypatch)
    assert "| chunk (of 256 tokens) |" in out and out.count("\n| ") >= 8 + 2 + 4
    assert "| bandwidth | 16-bit | 8-bit | 4-bit |" in out and "| 16 Gbps |" in out
    assert "| prompt tokens | compute-only s |" in out and "| 2048 |" in out
    out = _run(base + ["--grid", "--fluctuation", "--gbit", "8", "--shares", "0.5", "1.0"], capsys, monkeypatch)
    assert "| utilisation | compute-only s |" in out and "| 50.0 % |" in out and "| 100.0 % |" in out
    assert "fluctuation:" in out and "planned meet point" in out
