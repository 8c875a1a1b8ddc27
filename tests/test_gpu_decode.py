"""GPU parity of nsn_decode_attention against the oracle, on oracle-encoded caches (so the decode
check does not depend on the GPU encoder).  Tolerance: 2e-3 max relative error per output row
(max_i |out_i - ref_i| / max_i |ref_i|), fp32 accumulation on the device, fp64 in the oracle."""
import math

import numpy as np
import pytest

from oracle import nsn_oracle as O
from paper_2505_18231_amd import synth
from tests import helpers

pytestmark = pytest.mark.gpu
TOL = 2e-3


def build_case(seed, batch, hq, hkv, lens, sub, G, cb, page=0, max_len=None, per_seq=False):
    J = 128 // sub
    max_len = max_len or ((max(max(lens), 1) + 255) // 256) * 256
    bt = synth.shuffled_page_table(seed, batch, max_len // page) if page else None
    kc = helpers.HostCache("k", batch, hkv, J, max_len, G, page, bt)
    vc = helpers.HostCache("v", batch, hkv, J, max_len, G, page, bt)
    for b in range(batch):
        for h in range(hkv):
            if lens[b] == 0:
                continue
            kc.put_unit(b, h, O.encode(synth.make_k(seed, b, h, lens[b], per_seq=per_seq), cb, G))
            vc.put_unit(b, h, O.encode(synth.make_v(seed, b, h, lens[b]), cb, G))
    q = synth.make_q(seed, batch, hq)
    return kc, vc, q, max_len


def oracle_out(kc, vc, q, lens, hq, hkv, cb, G, scale):
    batch = q.shape[0]
    r = hq // hkv
    ref = np.zeros((batch, hq, 128))
    for b in range(batch):
        if lens[b] == 0:
            continue
        for h in range(hkv):
            ref[b, h * r:(h + 1) * r] = O.decode_attention(
                q[b, h * r:(h + 1) * r].astype(np.float64), kc.unit_dict(b, h, lens[b]),
                vc.unit_dict(b, h, lens[b]), cb, scale, G)
    return ref


def gpu_out(api, kc, vc, q, lens, hq, hkv, sub, G, cb, max_len, scale, page=0, n_splits=0):
    import torch
    shape = api.make_shape(sub, hq, hkv, max_len, G, page)
    dk, dv = kc.to_device(api, shape), vc.to_device(api, shape)
    cbd = torch.from_numpy(cb.astype(np.float16)).cuda()
    out = api.nsn_decode_attention(shape, cbd, torch.from_numpy(q).cuda(), dk, dv,
                                   torch.tensor(lens, dtype=torch.int32).cuda(), max(max(lens), 0), scale,
                                   n_splits)
    torch.cuda.synchronize()
    return out.cpu().numpy().astype(np.float64)


FLAT_LENS = [0, 1, 64, 65, 130, 300, 17, 256, 511, 77, 128, 5, 200, 333, 90, 400]
CASES = [
    # name, batch, hq, hkv, lens, sub, G, page, splits
    ("tiny-1bit", 1, 1, 1, [1024], 8, 0, 0, 0),
    ("tiny-1bit-1split", 1, 1, 1, [1024], 8, 0, 0, 1),
    ("tiny-1bit-3splits", 1, 1, 1, [1000], 8, 64, 0, 3),
    ("gqa-2bit-ragged", 2, 8, 2, [777, 130], 4, 64, 0, 4),
    ("gqa-2bit-onegroup", 2, 8, 2, [515, 1], 4, 0, 0, 0),
    ("mha-2bit", 2, 4, 4, [333, 700], 4, 64, 0, 2),
    ("paged-1bit", 3, 4, 2, [1000, 256, 37], 8, 0, 256, 0),
    ("paged-2bit-groups", 2, 8, 2, [900, 511], 4, 128, 256, 5),
    # more than 64 pages per sequence: a wave's window of block-table entries is reloaded on the way
    ("paged64-long-2bit", 2, 4, 2, [5000, 4200], 4, 64, 64, 3),
    ("paged192-long-1bit", 1, 4, 1, [13000], 8, 0, 192, 2),
    ("empty-and-short", 3, 2, 1, [0, 1, 65], 8, 64, 0, 2),
    ("gqa8-2bit", 1, 8, 1, [300], 4, 64, 0, 2),          # 8 query heads per kv head
    ("long-2bit-many-splits", 1, 4, 1, [5000], 4, 0, 0, 16),
    ("long-1bit-groups", 1, 4, 2, [3000], 8, 64, 0, 3),
    ("long-2bit-eleven-waves", 2, 4, 1, [9000, 4100], 4, 64, 0, 2),   # splits of >= 4096 tokens: the 11-wave instance
    ("long-2bit-eleven-waves-mha", 1, 1, 1, [5000], 4, 0, 0, 1),
    ("long-1bit-eleven-waves", 2, 4, 1, [9000, 4100], 8, 64, 0, 2),   # the 8-dim form of the 11-wave instance
    # 128 (sequence, kv head) units and automatic splitting: the persistent instance (equal runs of the list of
    # all 64-token groups; short units share a run, long ones are cut by run boundaries; empty sequences)
    ("flat-ragged-2bit", 16, 16, 8, FLAT_LENS, 4, 64, 0, 0),
    ("flat-paged-1bit", 16, 8, 8, FLAT_LENS[5:] + FLAT_LENS[:5], 8, 0, 256, 0),
    ("flat-gqa8-2bit-onegroup", 16, 64, 8, FLAT_LENS[::-1], 4, 0, 0, 0),
    ("flat-long-units-1bit", 16, 32, 8, [2100, 0, 70, 1500] + [40] * 12, 8, 128, 0, 0),
    # more than 64 sequences: the run boundaries are found across several 64-sequence blocks of lengths
    ("flat-paged64-long-1bit", 16, 8, 8, [4500, 0, 70, 5000] + [40] * 12, 8, 128, 64, 0),
    ("flat-all-empty", 16, 8, 8, [0] * 16, 4, 64, 0, 0),
    ("flat-130-sequences-1bit", 130, 2, 1, [(i * 37) % 200 for i in range(130)], 8, 0, 0, 0),
    ("flat-200-sequences-2bit-paged", 200, 4, 1, [(i * 53) % 300 for i in range(200)], 4, 64, 256, 0),
]


@pytest.mark.parametrize("impl", ["mfma", "lut"])
@pytest.mark.parametrize("name,batch,hq,hkv,lens,sub,G,page,splits", CASES, ids=[c[0] for c in CASES])
def test_decode_matches_oracle(gpu_api, codebooks, select_variant, impl, name, batch, hq, hkv, lens, sub, G, page,
                               splits):
    # "mfma": matrix-core kernel (default for <= 4 query heads per kv head); "lut": lookup-table kernel
    select_variant("decode", impl)
    print(f"case {name} impl={impl} lens={lens} sub={sub} G={G} page={page} splits={splits}", flush=True)
    cb = codebooks[sub]
    scale = 1.0 / math.sqrt(128)
    kc, vc, q, max_len = build_case(100 + len(name), batch, hq, hkv, lens, sub, G, cb, page)
    ref = oracle_out(kc, vc, q, lens, hq, hkv, cb, G, scale)
    out = gpu_out(gpu_api, kc, vc, q, lens, hq, hkv, sub, G, cb, max_len, scale, page, splits)
    for b in range(batch):
        if lens[b] == 0:
            assert np.all(out[b] == 0.0)
    live = [b for b in range(batch) if lens[b] > 0]
    if not live:
        return
    err = helpers.max_rel_err(out[live], ref[live])
    print(f"  max rel err {err:.3e}", flush=True)
    assert err < TOL, err


@pytest.mark.parametrize("impl", ["mfma", "lut"])
def test_split_count_does_not_change_the_result(gpu_api, codebooks, select_variant, impl):
    select_variant("decode", impl)
    cb = codebooks[4]
    scale = 1.0 / math.sqrt(128)
    lens = [1500, 640]
    kc, vc, q, max_len = build_case(7, 2, 8, 2, lens, 4, 64, cb)
    outs = [gpu_out(gpu_api, kc, vc, q, lens, 8, 2, 4, 64, cb, max_len, scale, 0, s) for s in (1, 2, 7)]
    # lut: fp32 everywhere, only the summation order changes.  mfma: the softmax weights enter the
    # value contraction as fp16 (relative 2^-11 each), and their rounding depends on the running max.
    tol = 2e-5 if impl == "lut" else 1e-3
    for o in outs[1:]:
        err = helpers.max_rel_err(o, outs[0])
        print(f"  split-count difference {err:.3e}", flush=True)
        assert err < tol


def _encoded_case(seed, hq, hkv, L, sub, G, cb, k_fn, v_fn):
    """One sequence whose keys / values come from k_fn(h), v_fn(h) (fp16 [L][128]), oracle-encoded."""
    J = 128 // sub
    max_len = ((L + 255) // 256) * 256
    kc = helpers.HostCache("k", 1, hkv, J, max_len, G)
    vc = helpers.HostCache("v", 1, hkv, J, max_len, G)
    for h in range(hkv):
        kc.put_unit(0, h, O.encode(k_fn(h), cb, G))
        vc.put_unit(0, h, O.encode(v_fn(h), cb, G))
    return kc, vc, synth.make_q(seed, 1, hq), max_len


@pytest.mark.parametrize("impl", ["mfma", "lut"])
@pytest.mark.parametrize("sub", [4, 8])
@pytest.mark.parametrize("log2_mul", [-12, 0, 9])
def test_value_scale_does_not_change_the_accuracy(gpu_api, codebooks, select_variant, impl, sub, log2_mul):
    """The first Normalize stores every token norm on its own (Sec. 3.2), so attention over the coded
    cache (App. B) is as accurate for values of size 2^-12 or 2^9 as for values of size 1."""
    select_variant("decode", impl)
    cb, scale, L, seed = codebooks[sub], 1.0 / math.sqrt(128), 1500, 60 + sub
    mul = np.float32(2.0 ** log2_mul)
    kc, vc, q, max_len = _encoded_case(
        seed, 8, 2, L, sub, 64, cb, lambda h: synth.make_k(seed, 0, h, L),
        lambda h: (synth.make_v(seed, 0, h, L).astype(np.float32) * mul).astype(np.float16))
    ref = oracle_out(kc, vc, q, [L], 8, 2, cb, 64, scale)
    out = gpu_out(gpu_api, kc, vc, q, [L], 8, 2, sub, 64, cb, max_len, scale, 0, 3)
    err = helpers.max_rel_err(out, ref)
    print(f"  impl={impl} sub={sub} V x 2^{log2_mul}: max rel err {err:.3e}, |ref| max {np.abs(ref).max():.3e}",
          flush=True)
    assert np.isfinite(out).all()
    assert err < TOL, err


@pytest.mark.parametrize("impl", ["mfma", "lut"])
@pytest.mark.parametrize("sub", [4, 8])
def test_sink_token_with_twice_the_norm(gpu_api, codebooks, select_variant, impl, sub):
    """Token 0 of the sequence is an outlier-norm ("sink") token: its key and its value are twice as
    long as they were drawn (Sec. 3.2 keeps such tokens apart through the stored norm)."""
    select_variant("decode", impl)
    cb, scale, L, seed = codebooks[sub], 1.0 / math.sqrt(128), 1100, 80 + sub

    def doubled(x):
        x = x.copy()
        x[0] = (x[0].astype(np.float32) * 2).astype(np.float16)
        return x
    for G in (0, 64):
        kc, vc, q, max_len = _encoded_case(seed, 4, 1, L, sub, G, cb,
                                           lambda h: doubled(synth.make_k(seed, 0, h, L)),
                                           lambda h: doubled(synth.make_v(seed, 0, h, L)))
        ref = oracle_out(kc, vc, q, [L], 4, 1, cb, G, scale)
        out = gpu_out(gpu_api, kc, vc, q, [L], 4, 1, sub, G, cb, max_len, scale, 0, 2)
        err = helpers.max_rel_err(out, ref)
        print(f"  impl={impl} sub={sub} G={G}: max rel err {err:.3e}", flush=True)
        assert err < TOL, err


@pytest.mark.parametrize("impl", ["mfma", "lut"])
@pytest.mark.parametrize("where", [0, 70001, 102399])
def test_one_dominant_token_among_many_low_score_tokens(gpu_api, codebooks, select_variant, impl, where):
    """102400 tokens whose scores are all near zero, and one token whose key points along the first
    query head (score about +17 after scaling): that head's softmax is almost one-hot, the running
    maximum jumps once, and the result must still be within the bar.  The cache is 2048 oracle-encoded
    tokens repeated 50 times (one Shift group, so repeated tokens encode identically)."""
    select_variant("decode", impl)
    sub, hq, L0, reps, seed = 4, 4, 2048, 50, 97
    cb, scale, J = codebooks[sub], 1.0 / math.sqrt(128), 32
    L = L0 * reps
    q = synth.make_q(seed, 1, hq)
    k = (synth.make_k(seed, 0, 0, L0).astype(np.float32) * np.float32(0.05)).astype(np.float16)
    v = synth.make_v(seed, 0, 0, L0)
    ek, ev = O.encode(k, cb, 0), O.encode(v, cb, 0)
    tiled_k = dict(codes=np.tile(ek["codes"], (reps, 1)), a=np.tile(ek["a"], reps), b=np.tile(ek["b"], reps), o=ek["o"])
    tiled_v = dict(codes=np.tile(ev["codes"], (reps, 1)), a=np.tile(ev["a"], reps), b=np.tile(ev["b"], reps), o=ev["o"])
    star = (q[0, 0].astype(np.float32) * np.float32(1.5)).astype(np.float16)[None, :]
    es = O.encode(star, cb, 0, start=where, frozen_o=ek["o"])
    for key in ("codes", "a", "b"):
        tiled_k[key][where] = es[key][0]
    kc = helpers.HostCache("k", 1, 1, J, L, 0)
    vc = helpers.HostCache("v", 1, 1, J, L, 0)
    kc.put_unit(0, 0, tiled_k)
    vc.put_unit(0, 0, tiled_v)
    ref = oracle_out(kc, vc, q, [L], hq, 1, cb, 0, scale)
    sc = O.lut_scores(q[0].astype(np.float64), kc.unit_dict(0, 0, L), cb, scale, 0)[0]
    weight = 1.0 / np.exp(sc - sc[where]).sum()
    assert weight > 0.9, weight
    out = gpu_out(gpu_api, kc, vc, q, [L], hq, 1, sub, 0, cb, L, scale, 0, 0)
    err = helpers.max_rel_err(out, ref)
    print(f"  impl={impl} dominant token at {where} (weight {weight:.4f}): max rel err {err:.3e}", flush=True)
    assert err < TOL, err


@pytest.mark.parametrize("seed", range(16))
def test_persistent_instance_agrees_with_forced_splits_on_random_shapes(gpu_api, seed):
    """The persistent instance (automatic split choice, 128 or more units) against the one-workgroup-per-split
    instance (forced split count), which the oracle cases above cover, on random batch shapes: ragged lengths
    with empty sequences, several kv-head counts, paged and contiguous caches, Shift groups, both code widths.
    Cache contents are random bytes (every byte is a valid code); the two launches differ in how the softmax
    partials are cut, so they agree to the rounding of the fp16 value weights, not bit for bit."""
    import torch
    api = gpu_api
    rng = np.random.default_rng(9000 + seed)
    hkv = int(rng.choice([1, 2, 4, 8]))
    r = int(rng.choice([1, 2, 4]))
    batch = int(rng.integers((128 + hkv - 1) // hkv, (128 + hkv - 1) // hkv + 40))
    sub = int(rng.choice([4, 8]))
    # (page size, Shift group size): powers of two and the general instances (192)
    page, G = [(0, 0), (0, 64), (0, 128), (0, 192), (64, 0), (64, 64), (256, 64), (256, 128), (256, 0),
               (192, 0)][int(rng.integers(0, 10))]
    top = int(rng.choice([90, 700, 3000]))
    lens = rng.integers(0, top, size=batch)
    lens[rng.integers(0, batch, size=3)] = 0
    lens[rng.integers(0, batch)] = top + 2000  # one long unit, cut by several run boundaries
    lens = [int(n) for n in lens]
    max_len = ((max(lens) + 767) // 768) * 768
    print(f"seed {seed}: batch={batch} hkv={hkv} r={r} sub={sub} page={page} G={G} top={top}", flush=True)
    shape = api.make_shape(sub, hkv * r, hkv, max_len, G, page)
    dev = torch.device("cuda")
    g = torch.Generator(device=dev).manual_seed(seed)
    bt = torch.from_numpy(synth.shuffled_page_table(seed, batch, max_len // page)).to(dev) if page else None
    caches = []
    for _ in range(2):
        c = api.alloc_cache(shape, batch, block_table=bt)
        c.codes.random_(0, 256, generator=g)
        c.norms.copy_((torch.rand(c.norms.shape, device=dev, generator=g) + 0.5).half())
        c.means.copy_((0.2 * torch.randn(c.means.shape, device=dev, generator=g)).half())
        caches.append(c)
    cb = torch.randn((256, sub), device=dev, generator=g).half()
    q = torch.randn((batch, hkv * r, 128), device=dev, generator=g).half()
    lens_d = torch.tensor(lens, dtype=torch.int32, device=dev)
    scale = 1.0 / math.sqrt(128)
    outs = []
    for n_splits in (0, 1, 3):
        o = api.nsn_decode_attention(shape, cb, q, caches[0], caches[1], lens_d, max(lens), scale, n_splits)
        torch.cuda.synchronize()
        outs.append(o.cpu().numpy().astype(np.float64))
    for b in range(batch):
        if lens[b] == 0:
            assert np.all(outs[0][b] == 0.0)
    assert np.all(np.isfinite(outs[0]))
    for o in outs[1:]:
        err = helpers.max_rel_err(outs[0], o)
        print(f"  difference to a forced split count {err:.3e}", flush=True)
        assert err < 1e-3, err


@pytest.mark.parametrize("sub,page", [(4, 0), (8, 0), (4, 64)])
def test_smallest_cache_one_group(gpu_api, codebooks, sub, page):
    """A cache of a single 64-token group per array (the smallest the layout allows): the loads that the kernel
    issues for groups past the end of a wave's list read the first bytes of each array and must stay inside it."""
    cb = codebooks[sub]
    scale = 1.0 / math.sqrt(128)
    lens = [37]
    kc, vc, q, max_len = build_case(4242, 1, 1, 1, lens, sub, 0, cb, page, max_len=64)
    assert max_len == 64
    ref = oracle_out(kc, vc, q, lens, 1, 1, cb, 0, scale)
    out = gpu_out(gpu_api, kc, vc, q, lens, 1, 1, sub, 0, cb, max_len, scale, page)
    err = helpers.max_rel_err(out, ref)
    print(f"  sub={sub} page={page}: max rel err {err:.3e}", flush=True)
    assert err < TOL, err


@pytest.mark.parametrize("seed", range(12))
def test_matrix_core_and_lookup_table_kernels_agree_on_random_shapes(gpu_api, select_variant, seed):
    """The default (matrix-core) decode kernel against the lookup-table kernel, which computes the same sums in
    fp32 with scalar arithmetic and shares no code with it, on random small batch shapes: 1 to 8 query heads per
    kv head, forced and automatic split counts, paged and contiguous caches, Shift groups, both code widths.
    Cache contents are random bytes (every byte is a valid code)."""
    import torch
    api = gpu_api
    rng = np.random.default_rng(7000 + seed)
    hkv = int(rng.choice([1, 2, 4]))
    r = int(rng.choice([1, 2, 3, 4, 8]))
    batch = int(rng.integers(1, 7))
    sub = int(rng.choice([4, 8]))
    page, G = [(0, 0), (0, 64), (0, 128), (0, 192), (64, 0), (64, 64), (256, 64), (256, 128), (256, 0),
               (192, 0)][int(rng.integers(0, 10))]
    n_splits = int(rng.choice([0, 0, 1, 2, 3, 5, 9]))
    lens = [int(n) for n in rng.integers(0, 3000, size=batch)]
    lens[int(rng.integers(0, batch))] = int(rng.integers(1, 6000))  # at least one sequence with tokens
    max_len = ((max(lens) + 767) // 768) * 768
    print(f"seed {seed}: batch={batch} hkv={hkv} r={r} sub={sub} page={page} G={G} splits={n_splits} lens={lens}", flush=True)
    shape = api.make_shape(sub, hkv * r, hkv, max_len, G, page)
    dev = torch.device("cuda")
    g = torch.Generator(device=dev).manual_seed(seed)
    bt = torch.from_numpy(synth.shuffled_page_table(seed, batch, max_len // page)).to(dev) if page else None
    caches = []
    for _ in range(2):
        c = api.alloc_cache(shape, batch, block_table=bt)
        c.codes.random_(0, 256, generator=g)
        c.norms.copy_((torch.rand(c.norms.shape, device=dev, generator=g) + 0.5).half())
        c.means.copy_((0.2 * torch.randn(c.means.shape, device=dev, generator=g)).half())
        caches.append(c)
    cb = torch.randn((256, sub), device=dev, generator=g).half()
    q = torch.randn((batch, hkv * r, 128), device=dev, generator=g).half()
    lens_d = torch.tensor(lens, dtype=torch.int32, device=dev)
    scale = 1.0 / math.sqrt(128)
    outs = {}
    for impl in ("mfma", "lut"):
        select_variant("decode", impl)
        o = api.nsn_decode_attention(shape, cb, q, caches[0], caches[1], lens_d, max(lens), scale, n_splits)
        torch.cuda.synchronize()
        outs[impl] = o.cpu().numpy().astype(np.float64)
    for b in range(batch):
        if lens[b] == 0:
            assert np.all(outs["mfma"][b] == 0.0)
    assert np.all(np.isfinite(outs["mfma"]))
    err = helpers.max_rel_err(outs["mfma"], outs["lut"])
    print(f"  difference between the two kernels {err:.3e}", flush=True)
    assert err < TOL, err
