"""Host-side pieces that need no GPU: the bench's command line contract and the input recipes."""
import os
import subprocess
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "ONE GPU" in (r.stderr + r.stdout)


def test_input_recipes_are_seeded_and_shaped():
    import obc_inputs

    for name, spec in obc_inputs.SPECS.items():
        if spec.d_col > 600:
            continue                      # the large layers are generated on the GPU machine only
        W1, X1, s1 = obc_inputs.make_layer(name, device="cpu", n_samples=min(spec.n_samples, 512))
        W2, X2, _ = obc_inputs.make_layer(name, device="cpu", n_samples=min(spec.n_samples, 512))
        assert W1.shape == (spec.d_row, spec.d_col) and X1.shape[0] == spec.d_col
        assert np.array_equal(W1.numpy(), W2.numpy()) and np.array_equal(X1.numpy(), X2.numpy())
        assert np.isfinite(X1.numpy()).all() and np.isfinite(W1.numpy()).all()
    assert obc_inputs.target_count(0.5, 16, 32) == 256
    assert obc_inputs.target_count(0.6, 64, 576) == int(0.6 * 64 * 576)
