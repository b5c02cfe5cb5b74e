"""The race-hunting build (a workgroup fence after every phase of the forward and every tile or step of the
backward kernels) against the release build: same arithmetic in the same order, so every output must agree
bit for bit.  A difference would mean the release build reads a tile buffer that is being refilled, or the
other way round."""
import os
import subprocess
import sys
import tempfile

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

# (lengths, pack_len, Hq, Hkv, d_qk, d_v): several tiles per sample and ragged tails, both forward
# workgroup shapes (even and odd group sizes), all three head sizes, the wrapped block order of long samples
CASES = [
    ([512, 256, 128, 64, 64], 1024, 4, 4, 64, 64),
    ([1, 2, 31, 32, 33, 63, 64, 65, 127, 128, 129, 200, 257, 5, 300], 1407, 4, 1, 128, 128),
    ([700, 129, 256, 257, 31, 1, 400], 1774, 3, 3, 128, 128),
    ([900, 333, 1], 1234, 2, 2, 192, 128),
    ([5197, 300], 5497, 8, 8, 64, 64),
    ([3000, 700, 130], 3830, 16, 4, 128, 128),
]

RUNNER = r"""
import sys, numpy as np
sys.path.insert(0, %(root)r); sys.path.insert(0, %(tests)r)
from parity_util import Case, run_gpu
import paper_2503_07680_amd as H
cases = %(cases)r
out = {}
for i, (lengths, pack_len, Hq, Hkv, d, e) in enumerate(cases):
    pa, dev, res = run_gpu(Case(lengths, pack_len, Hq, Hkv, d, e, seed=80 + i, name="racehunt-%%d" %% i))
    for k, v in res.items():
        out["%%d_%%s" %% (i, k)] = v
    print("case", i, "done with", H.library_path(), flush=True)
np.savez(sys.argv[1], **out)
"""


def run_with(library, path):
    env = dict(os.environ)
    if library:
        env["HBP_LIBRARY"] = library
    else:
        env.pop("HBP_LIBRARY", None)
    code = RUNNER % {"root": ROOT, "tests": os.path.join(ROOT, "tests"), "cases": CASES}
    r = subprocess.run([sys.executable, "-c", code, path], env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT,
                       text=True, timeout=600)
    assert r.returncode == 0, r.stdout[-3000:]
    assert ("libhbp_racehunt.so" in r.stdout) == bool(library), r.stdout[-500:]
    return np.load(path)


def test_release_and_race_hunting_builds_agree_bit_for_bit():
    from paper_2503_07680_amd import build as B
    assert os.path.exists(B.LIB_RACE_HUNT), "build the library first (python -m paper_2503_07680_amd.build)"
    with tempfile.TemporaryDirectory() as tmp:
        release = run_with(None, os.path.join(tmp, "release.npz"))
        fenced = run_with("libhbp_racehunt.so", os.path.join(tmp, "fenced.npz"))
        assert sorted(release.files) == sorted(fenced.files) and len(release.files) == 5 * len(CASES)
        for name in release.files:
            assert np.array_equal(release[name].view(np.uint32), fenced[name].view(np.uint32)), name
