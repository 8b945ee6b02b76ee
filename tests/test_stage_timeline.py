"""The per-stage timeline tool: its event parsing on fabricated events (CPU), and one real run on the
tiny workload (GPU)."""
import sys

import numpy as np
import pytest

from paper_2404_16710_amd import stage_timeline as ST


def _fake_layer(t0, attention=True):
    """(time, tag) events of one layer starting at t0 (microseconds), 1 us apart."""
    tags = [0x10, 0x11, 0x12, 0x13, 0x80, 0x81, 0x14, 0x15, 0x16,
            0x20, 0x22] + ([0x23, 0x24, 0x27, 0x28, 0x29, 0x25] if attention else []) + [0x26,
            0x30, 0x31, 0x32, 0x80, 0x81, 0x34, 0x35, 0x36,
            0x40, 0x41, 0x42, 0x43, 0x80, 0x81, 0x44, 0x80, 0x81, 0x44, 0x45, 0x46,
            0x50, 0x51, 0x52, 0x80, 0x81, 0x54, 0x55, 0x56]
    return [(t0 + i, g) for i, g in enumerate(tags)]


def test_layers_are_cut_at_stage_starts_and_split_by_pass_kind():
    ev = [(0.0, 0x90)]
    for k in range(3):
        ev += _fake_layer(10.0 + 100.0 * k)
    ev += [(400.0, 0x60), (401.0, 0x70), (402.0, 0x76), (403.0, 0x91)]
    for k in range(3):
        ev += _fake_layer(410.0 + 200.0 * k)
    t = np.array([e[0] for e in ev]); tag = np.array([e[1] for e in ev])
    times, pattern, layer_us = ST._layers(t, tag, 0x90)
    assert layer_us == 100.0 and pattern[0] == 0x10 and len(times) == len(pattern)
    times2, pattern2, layer_us2 = ST._layers(t, tag, 0x91)
    assert layer_us2 == 200.0 and pattern2 == pattern
    rows = ST._stage_table(times, pattern, [1e6, 0, 2e6, 3e6, 4e6], layer_us)
    assert len(rows) == 2 + len(ST.STAGES)
    qkv = rows[2].split("|")
    # QKV: barrier 0x10 -> 0x12 = 2 us, input fetch 0x12 -> 0x80 = 2 us, stream 0x80 -> 0x81 = 1 us
    assert [x.strip() for x in qkv[3:6]] == ["2.00", "2.00", "1.00"]
    assert "(q, K, V)" in rows[3]
    none = ST._layers(t[:5], tag[:5], 0x91)
    assert none == (None, None, None)


def test_a_workgroup_without_an_attention_item_is_reported_as_such():
    ev = [(0.0, 0x90)]
    for k in range(3):
        ev += _fake_layer(10.0 + 100.0 * k, attention=False)
    t = np.array([e[0] for e in ev]); tag = np.array([e[1] for e in ev])
    times, pattern, layer_us = ST._layers(t, tag, 0x90)
    rows = ST._stage_table(times, pattern, [1e6, 0, 2e6, 3e6, 4e6], layer_us)
    assert "no attention item" in rows[3]


@pytest.mark.gpu
def test_timeline_of_the_tiny_workload(monkeypatch, capsys):
    monkeypatch.setattr(sys, "argv", ["stage_timeline", "--config", "c1", "--workgroup", "0"])
    ST.main()
    out = capsys.readouterr().out
    assert "one-row pass" in out and "| QKV + RoPE + cache append |" in out and "head and pass overhead" in out
