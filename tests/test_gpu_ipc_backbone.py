"""Zero-copy shared backbone across processes (paper sections 4.4, 5, 6.9): one process holds W0 and exports an
inter-process memory handle, two other processes map it and run the multi-LoRA layer on the mapped pointer with their
own adapters; each result is checked against the oracle inside that process, and the holder verifies that W0 is
bit-for-bit what it wrote.  All three are fresh child processes of the test (none replaces itself after touching
the GPU)."""
import json
import os
import subprocess
import sys
import tempfile

import pytest

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_two_functions_share_one_backbone_through_an_ipc_handle():
    script = os.path.join(ROOT, "tests", "ipc_roles.py")
    env = dict(os.environ, HSA_ENABLE_IPC_MODE_LEGACY="0")
    with tempfile.TemporaryDirectory() as d:
        procs = [subprocess.Popen([sys.executable, "-u", script, "holder", d, "2"], env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)]
        procs += [subprocess.Popen([sys.executable, "-u", script, "client", d, str(i)], env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
                  for i in range(2)]
        outs = []
        try:
            for p in procs:
                out, _ = p.communicate(timeout=200)
                outs.append(out)
        finally:
            for p in procs:
                if p.poll() is None:
                    p.kill()
        for p, out in zip(procs, outs):
            assert p.returncode == 0, out[-2000:]
        assert json.load(open(os.path.join(d, "holder.json")))["unchanged"] is True
        for i in range(2):
            r = json.load(open(os.path.join(d, f"client_{i}.json")))
            assert r["err_over_rms"] <= 2e-2
            # the mapping duplicates nothing: a small fraction of the 4 MiB it maps, at most
            assert r["device_bytes_taken_by_the_mapping"] <= r["backbone_bytes"] // 2, r
            print(f"client {i}: err/rms {r['err_over_rms']:.2e}, open {r['open_ms']:.3f} ms, "
                  f"device bytes taken by the mapping {r['device_bytes_taken_by_the_mapping']}", flush=True)
