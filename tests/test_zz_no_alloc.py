"""The entry point that allocates nothing (nsn_decode_attention_noalloc: scratch in a fixed array of the
library) gives the same output as nsn_decode_attention, on two calls in a row, the second smaller."""
import math

import numpy as np
import pytest

from paper_2505_18231_amd import synth
from tests import helpers
from tests.test_gpu_decode import build_case

pytestmark = pytest.mark.gpu


def _both(api, cb, seed, batch, hq, hkv, lens, sub, G, splits):
    import torch
    scale = 1.0 / math.sqrt(128)
    kc, vc, q, max_len = build_case(seed, batch, hq, hkv, lens, sub, G, cb)
    shape = api.make_shape(sub, hq, hkv, max_len, G)
    dk, dv = kc.to_device(api, shape), vc.to_device(api, shape)
    cbd = torch.from_numpy(cb.astype(np.float16)).cuda()
    qd = torch.from_numpy(q).cuda()
    ld = torch.tensor(lens, dtype=torch.int32).cuda()
    ref = api.nsn_decode_attention(shape, cbd, qd, dk, dv, ld, max(lens), scale, splits)
    out = torch.full((batch, hq, 128), float("nan"), dtype=torch.float32, device="cuda")
    api.nsn_decode_attention_noalloc(shape, cbd, qd, dk, dv, ld, max(lens), scale, splits, out=out)
    torch.cuda.synchronize()
    return out.cpu().numpy(), ref.cpu().numpy()


def test_noalloc_matches_workspace_entry_point_twice(gpu_api, codebooks):
    # first call: 2 sequences x 8 query heads, 5 splits; second call: smaller in every size
    out, ref = _both(gpu_api, codebooks[4], 31, 2, 8, 2, [1500, 640], 4, 64, 5)
    print(f"call 1: max abs diff {np.abs(out - ref).max():.3e}", flush=True)
    assert np.array_equal(out, ref)          # same kernels, same order of operations: bit-identical
    out, ref = _both(gpu_api, codebooks[8], 32, 1, 4, 1, [300], 8, 0, 2)
    print(f"call 2: max abs diff {np.abs(out - ref).max():.3e}", flush=True)
    assert np.array_equal(out, ref)


def test_noalloc_persistent_instance_matches_workspace_entry_point(gpu_api, codebooks):
    # 16 sequences x 8 kv heads = 128 units with automatic splitting: the persistent instance, whose partials
    # (two per run) and counters live in the same scratch array
    lens = [0, 1, 64, 65, 130, 300, 17, 256, 511, 77, 128, 5, 200, 333, 90, 400]
    out, ref = _both(gpu_api, codebooks[4], 33, 16, 16, 8, lens, 4, 64, 0)
    assert np.array_equal(out, ref)
    out, ref = _both(gpu_api, codebooks[4], 34, 2, 8, 2, [700, 100], 4, 64, 3)   # then a small split call again
    assert np.array_equal(out, ref)


def test_noalloc_rejects_calls_beyond_its_scratch(gpu_api, codebooks):
    import torch
    api = gpu_api
    shape = api.make_shape(4, 32, 8, 8192, 0)
    # 64 sequences x 32 heads x 4 splits x 1032 bytes = 8.5 MB > 4 MiB
    kc, vc = api.alloc_cache(shape, 1), api.alloc_cache(shape, 1)
    q = torch.zeros((64, 32, 128), dtype=torch.float16, device="cuda")
    out = torch.zeros((64, 32, 128), dtype=torch.float32, device="cuda")
    lens = torch.zeros(64, dtype=torch.int32, device="cuda")
    cb = torch.zeros((256, 4), dtype=torch.float16, device="cuda")
    with pytest.raises(api.NsnError) as e:
        api.nsn_decode_attention_noalloc(shape, cb, q, kc, vc, lens, 8192, 0.1, 4, out=out)
    assert e.value.code == api.NSN_ERR_WORKSPACE
