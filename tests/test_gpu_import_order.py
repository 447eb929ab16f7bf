"""The library must work whichever of the package and PyTorch a program imports first."""
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

CODE = r"""
import sys
sys.path.insert(0, %r)
sys.path.insert(0, %r)
import numpy as np
import paper_2204_03643_amd as tv
assert "stream_bytes" in tv.tv_dispatch_thresholds()      # loads libtvprox.so
assert "torch" in sys.modules, "the binding imports PyTorch ahead of the library"
import torch
import oracle
rng = np.random.default_rng(3)
y = rng.normal(size=(300, 32)).astype(np.float32)
lam = np.array([0.4], np.float32)
yt = torch.from_numpy(y).cuda()
lt = torch.from_numpy(lam).cuda()
xt = torch.full_like(yt, float("nan"))
tv.tv1d_prox_fwd(yt, xt, tv.rows_along(y.shape, -1), tv.tv_lambda(lt.data_ptr(), 1, 1))
torch.cuda.synchronize()
ref = oracle.prox1d_batch(y.astype(np.float64), lam.astype(np.float64))
err = np.abs(xt.cpu().numpy() - ref).max() / (1 + np.abs(y).max())
assert err <= 1e-4, err
print("ok")
"""


def test_package_imported_and_library_loaded_before_torch():
    """A fresh interpreter imports the package, makes it load the library, and only then imports
    PyTorch: the forward call must run and match the oracle (it failed with a HIP error when the
    library pulled in the system's HIP runtime ahead of PyTorch's own)."""
    res = subprocess.run([sys.executable, "-c", CODE % (ROOT, os.path.join(ROOT, "tests"))], capture_output=True,
                         text=True, timeout=300, cwd=ROOT)
    assert res.returncode == 0 and "ok" in res.stdout, res.stdout[-2000:] + res.stderr[-2000:]
