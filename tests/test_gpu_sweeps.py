"""The sweep tool end to end on a small shape: every mode prints its table, and one number per mode is
checked that the method fixes whatever the host's timing (paced load times, token and chunk counts)."""
import re
import sys

import pytest

pytestmark = pytest.mark.gpu


def _run(argv, capsys, monkeypatch):
    from paper_2410_03065_amd import sweeps
    monkeypatch.setattr(sys, "argv", ["sweeps"] + argv)
    sweeps.main()
    return capsys.readouterr().out


def _rows(out, header):
    """Cells of the table whose header line starts with `header`."""
    lines = out.splitlines()
    i = next(k for k, l in enumerate(lines) if l.startswith(header))
    rows = []
    for l in lines[i + 2:]:
        if not l.startswith("| "):
            break
        rows.append([c.strip() for c in l.strip("|").split("|")])
    return rows


def test_sweep_tables_on_a_small_shape(capsys, monkeypatch):
    # tiny float32 shape: 4 KiB of KV per token, so a 256-token chunk is 1 MiB and the prompt 8 MiB
    base = ["--shape", "tiny-f32", "--tokens", "2048", "--budget", "256", "--fetch-unit", "64"]
    out = _run(base + ["--chunks", "--compression", "--lengths", "--gbit", "8", "16"], capsys, monkeypatch)
    # per-chunk table: eight chunks; a loaded chunk takes its bytes over the tier's rate (1 GB/s: 1.049 ms), paced,
    # never less, and computing a chunk reports a positive rate
    rows = _rows(out, "| chunk (of 256 tokens) |")
    assert [int(r[0]) for r in rows] == list(range(8))
    for r in rows:
        assert 1.048 <= float(r[3]) <= 1.048 * 1.25, r
        assert float(r[1]) > 0
    # compression table: one row per bandwidth, three stores, every meet point inside the prompt
    rows = _rows(out, "| bandwidth | 16-bit | 8-bit | 4-bit |")
    assert [r[0] for r in rows] == ["8 Gbps", "16 Gbps"]
    for r in rows:
        ms = [int(re.search(r"m=(\d+)", c).group(1)) for c in r[1:]]
        assert len(ms) == 3 and all(0 <= m <= 8 for m in ms), r
    # length table: quarters of the prompt, two to eight chunks, and the split never outside the prompt
    rows = _rows(out, "| prompt tokens | compute-only s |")
    assert [int(r[0]) for r in rows] == [512, 1024, 1536, 2048]
    for r, n in zip(rows, (2, 4, 6, 8)):
        for c in r[2:]:
            m, tot = map(int, re.search(r"(\d+)/(\d+)$", c).groups())
            assert tot == n and 0 <= m <= n, r
    out = _run(base + ["--grid", "--fluctuation", "--gbit", "8", "--shares", "0.5", "1.0"], capsys, monkeypatch)
    rows = _rows(out, "| utilisation | compute-only s |")
    assert [r[0] for r in rows] == ["50.0 %", "100.0 %"]
    for r in rows:      # tokens computed by the request: whole fetch units, inside the prompt
        m = int(re.search(r"m=(\d+)", r[2]).group(1))
        assert m % 64 == 0 and 0 <= m <= 2048, r
    # load-only: 8 MiB over 1 GB/s, paced (8.39 ms), whatever the host does
    t_l = float(re.search(r"load-only s: 8 Gbps ([0-9.]+)", out).group(1))
    assert 0.00838 <= t_l <= 0.00838 * 1.25, t_l
    m = re.search(r"fluctuation:.* (\d+) tokens computed, (\d+) loaded", out)
    assert int(m.group(1)) + int(m.group(2)) == 2048
    assert "planned meet point" in out
