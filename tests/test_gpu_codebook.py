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


@pytest.mark.parametrize("sub,n,iters,lr", [(4, 1 << 14, 6, 128.0), (8, 1 << 13, 4, 256.0)])
def test_finetune_matches_oracle_and_raises_cosine(gpu_api, sub, n, iters, lr):
    """nsn_finetune_codebook (Sec. 3.4) against the oracle's gradient steps from the same start."""
    import torch
    print(f"case sub={sub} n={n} iters={iters} lr={lr}", flush=True)
    samples = synth.codebook_samples(56, n, sub)
    start, _, _ = O.build_codebook(samples, 256, 3)
    ref, hist, ref_final = O.finetune_codebook(samples, start, iters, lr)
    cbd = torch.from_numpy(start.astype(np.float16)).cuda()
    cb, cos0, cos1 = gpu_api.nsn_finetune_codebook(torch.from_numpy(samples).cuda(), cbd, iters, lr)
    got = cb.cpu().numpy()
    diff = np.abs(got.view(np.int16).astype(np.int32) - ref.astype(np.float16).view(np.int16).astype(np.int32))
    print(f"  cosine {cos0:.6f} -> {cos1:.6f} (oracle {hist[0]:.6f} -> {ref_final:.6f}), "
          f"{(diff != 0).sum()} of {diff.size} fp16 entries differ, max {diff.max()} ulp", flush=True)
    assert diff.max() <= 1 and (diff == 0).mean() > 0.995
    assert abs(cos0 - hist[0]) < 1e-12
    assert abs(cos1 - ref_final) < 1e-9 + 1e-5 * (diff.max() > 0)
    assert cos1 > cos0 + 1e-4
    # zero steps: the codebook is returned unchanged
    same, c0, c1 = gpu_api.nsn_finetune_codebook(torch.from_numpy(samples).cuda(), cbd.clone(), 0, lr)
    assert torch.equal(same, cbd) and c0 == c1


@pytest.mark.parametrize("sub", [4, 8])
def test_codebook_on_16_levels_matches_oracle(gpu_api, codebooks, sub):
    import torch
    cb = codebooks[sub]
    want, code, mn, st = O.quantize_codebook_4bit(cb)
    got, codes, levels = gpu_api.nsn_quantize_codebook(torch.from_numpy(cb.astype(np.float16)).cuda())
    torch.cuda.synchronize()
    assert np.array_equal(got.cpu().numpy().astype(np.float64), want)
    assert np.array_equal(codes.cpu().numpy(), code)
    lv = levels.cpu().numpy()
    assert lv[0] == mn and lv[1] == st
