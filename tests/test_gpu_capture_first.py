"""The data-path calls are legal under stream capture from their very first use: a fresh process
captures the graph before any eager call (so every kernel's one-time set-up happens while the
stream is capturing), replays it, and compares with an eager run."""
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

PROGRAM = r"""
import torch
import synth
from synth.resident import ResidentLayer

for name, kw in (("c3", dict(T=900, H=512, I=256, I_shared=256)), ("c1", dict())):
    cfg = synth.scaled(synth.get_config(name), **kw)
    g = ResidentLayer(cfg, device="cuda:0")
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        g.capture(stream, overlap_shared=False)
        g.replay(stream)
        stream.synchronize()
        out_graph = g.buf["out"].clone()
        phys_graph = g.buf["topk_phys"].clone()
        g.buf["out"].zero_()
        g.forward(stream=stream, overlap_shared=False)
        stream.synchronize()
    assert torch.equal(phys_graph, g.buf["topk_phys"]), name
    assert torch.equal(out_graph, g.buf["out"]), name
    assert bool(torch.isfinite(out_graph.float()).all()) and float(out_graph.float().abs().sum()) > 0, name
    g.close()
print("capture-first ok")
"""


def test_capture_as_the_first_use_in_a_fresh_process():
    env = dict(os.environ, PYTHONPATH=ROOT + os.pathsep + os.environ.get("PYTHONPATH", ""))
    r = subprocess.run([sys.executable, "-c", PROGRAM], cwd=ROOT, env=env, capture_output=True, text=True, timeout=150)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "capture-first ok" in r.stdout
