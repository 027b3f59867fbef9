"""Host-side checks of bench.py that need no GPU: the one-GPU rule and the byte accounting."""
import os
import subprocess
import sys

import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and "--gpus 1" in r.stderr
    assert r.stdout.strip() == ""                      # no JSON line that could be mistaken for a measurement


def test_expert_bytes_match_the_shapes():
    sys.path.insert(0, ROOT)
    import bench
    cfg = wl.CONFIGS["mixtral"]
    gu, dn = bench.expert_bytes(cfg, 4)
    assert gu == 4 * 2 * 4096 * 14336 * 2 and dn == 4 * 4096 * 14336 * 2
    cfg = wl.CONFIGS["dsv2lite"]
    gu, dn = bench.expert_bytes(cfg, 10)
    per_expert = 3 * cfg.H * cfg.F * 2
    assert gu + dn == 10 * per_expert + cfg.n_shared * 3 * cfg.H * cfg.F_shared * 2


def test_layer_policy_table():
    sys.path.insert(0, ROOT)
    import pytest

    import bench
    names = bench.layer_policy("0-3:off,4-43:aggressive,44-47:moderate", 48, "aggressive")
    assert names[:4] == ["off"] * 4 and names[4:44] == ["aggressive"] * 40 and names[44:] == ["moderate"] * 4
    assert bench.layer_policy("", 3, "moderate") == ["moderate"] * 3          # layers not named keep the preset
    assert bench.layer_policy("2:off", 4, "moderate") == ["moderate", "moderate", "off", "moderate"]
    for bad in ("0-9:off", "1:sometimes", "3-1:off"):
        with pytest.raises(ValueError):
            bench.layer_policy(bad, 4, "off")
