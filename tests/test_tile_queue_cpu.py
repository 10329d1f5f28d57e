"""Host-side sweep of the persistent kernels' tile orders and queue shares (tests/tile_queue_driver.hip):
the integer functions the kernels use on the device are compiled for the host as well and checked to hand out
every tile exactly once, for both orders and several thousand tile counts.  CPU only."""
import os
import shutil
import subprocess

import pytest

from paper_2602_05885_amd import build as pgbuild

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("hipcc") is None and not os.path.exists("/opt/rocm/bin/hipcc"), reason="needs hipcc")
def test_every_tile_is_handed_out_exactly_once(tmp_path):
    exe = str(tmp_path / "tile_queue_driver")
    flags = [f for f in pgbuild.FLAGS if f not in ("-fPIC",)]
    subprocess.run([pgbuild.hipcc(), *flags, os.path.join(ROOT, "tests", "tile_queue_driver.hip"), "-o", exe],
                   check=True, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300)
    r = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=120)
    assert r.returncode == 0 and "(0 failures)" in r.stdout, r.stdout[-2000:]
