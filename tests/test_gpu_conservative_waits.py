"""The library against a build of the same sources in which every hand-counted wait of the contraction core is a
full wait and the untracked LDS accessors wait for everything in flight (`-DDSMOE_CONSERVATIVE_WAITS`,
libdsmoe_checked.so, built by paper_2404_05567_amd/build.py next to libdsmoe.so): the outputs must agree bit for bit
on every shape class of tests/hazard_probe.py.  A wait that let a stale LDS stage or an unfinished load through would
show here as a difference."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run_probe(library):
    env = dict(os.environ)
    if library:
        env["DSMOE_LIBRARY"] = library
    else:
        env.pop("DSMOE_LIBRARY", None)
    print(f"[case] hazard probe with {library or 'libdsmoe.so'}", flush=True)
    p = subprocess.run([sys.executable, "-u", os.path.join(ROOT, "tests", "hazard_probe.py")], env=env, cwd=ROOT,
                       capture_output=True, text=True, timeout=280)
    assert p.returncode == 0, p.stdout[-2000:] + p.stderr[-2000:]
    line = [l for l in p.stdout.splitlines() if l.startswith("DIGESTS ")][-1]
    return json.loads(line[len("DIGESTS "):])


def test_counted_waits_agree_with_full_waits_bit_for_bit():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2404_05567_amd as dsmoe
    if not os.path.exists(dsmoe.LIB_CHECKED_PATH):
        pytest.fail(f"{dsmoe.LIB_CHECKED_PATH} is missing: run `python -m paper_2404_05567_amd.build`")
    fast = run_probe(None)
    again = run_probe(None)
    checked = run_probe(dsmoe.LIB_CHECKED_PATH)
    assert len(fast) >= 18
    assert fast == again, {k: (fast[k], again[k]) for k in fast if fast[k] != again.get(k)}
    assert fast == checked, {k: (fast[k], checked[k]) for k in fast if fast[k] != checked.get(k)}
