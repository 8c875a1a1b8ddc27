"""GPU parity of nsn_build_codebook against the oracle's Lloyd iterations on the same samples."""
import numpy as np
import pytest

from oracle import nsn_oracle as O
from paper_2505_18231_amd import synth

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("sub,n,iters", [(8, 1 << 14, 5), (4, 1 << 15, 4), (4, 3000, 3)])
def test_codebook_matches_oracle(gpu_api, sub, n, iters):
    import torch
    print(f"case sub={sub} n={n} iters={iters}", flush=True)
    samples = synth.codebook_samples(55, n, sub)
    ref, _, ref_mse = O.build_codebook(samples, 256, iters)
    cb, mse = gpu_api.nsn_build_codebook(torch.from_numpy(samples).cuda(), 256, iters)
    got = cb.cpu().numpy()
    # both are single fp16 roundings of fp64 centroids that differ only by summation order
    diff = np.abs(got.view(np.int16).astype(np.int32) - ref.astype(np.float16).view(np.int16).astype(np.int32))
    assert diff.max() <= 1
    assert (diff == 0).mean() > 0.999
    assert abs(mse - ref_mse) < 1e-9 * max(ref_mse, 1.0) + 1e-6 * (diff.max() > 0)
