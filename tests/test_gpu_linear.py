"""The MFMA projection y = x w against fp64 numpy, ragged shapes included."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("n,fin,fout", [(1, 1, 1), (127, 15, 16), (129, 17, 65), (1000, 602, 256),
                                        (513, 500, 64), (300, 64, 192), (2049, 33, 130)])
def test_linear(n, fin, fout):
    import paper_2110_09524_amd as pk
    import torch
    from gpu_harness import assert_close, dev, empty
    print(f"linear: {n}x{fin}x{fout}", flush=True)
    rng = np.random.default_rng(n + fin + fout)
    x = rng.standard_normal((n, fin)).astype(np.float32)
    w = (rng.standard_normal((fin, fout)) / np.sqrt(fin)).astype(np.float32)
    y = empty((n, fout))
    pk.gnn_linear_fwd(dev(x), dev(w), y)
    torch.cuda.synchronize()
    assert_close("y", y.cpu().numpy(), x.astype(np.float64) @ w.astype(np.float64))
