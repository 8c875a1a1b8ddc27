"""GPU parity for keys normalised before the rotary embedding (Sec. 3.2 "NSN applied to key and
value", App. B): the encoder turns v_nsn by the token's position before the Hadamard rotation, the
attention kernel turns the stored mean inside the score.  Same bars as the plain path: codes
bit-exact outside the oracle's tie window, a within one fp16 ulp, attention rows within 2e-3."""
import math

import numpy as np
import pytest

from oracle import nsn_oracle as O
from paper_2505_18231_amd import synth
from tests import helpers
from tests.test_gpu_encode import check_unit, run_gpu_encode

pytestmark = pytest.mark.gpu
TOL = 2e-3
MAX_POS = 131072


@pytest.fixture(scope="module", params=[10000.0, 500000.0], ids=["base1e4", "base5e5"])
def rope(request, gpu_api):
    import torch
    f = synth.rope_inv_freq(request.param)
    table = gpu_api.nsn_build_rope_table(f, MAX_POS)
    torch.cuda.synchronize()
    return f, table


@pytest.fixture(scope="module")
def magnitude_codebook():
    x = np.abs(synth.codebook_samples(4242, 1 << 13, 8).astype(np.float64))
    cb, _, _ = O.build_codebook(x, 256, 5)
    return cb


def test_rope_table_against_fp64_cosines(gpu_api, rope):
    f, table = rope
    raw = table.cpu().numpy()
    f64 = f.astype(np.float64)
    j = np.arange(64)[:, None] * f64[None, :]
    want = np.concatenate([np.cos(j), np.sin(j)], axis=1)                       # [64][128]
    hi = raw[:16384].view(np.float16).reshape(64, 128).astype(np.float64)
    lo = raw[16384:32768].view(np.float16).reshape(64, 128).astype(np.float64)
    assert np.abs(hi - want).max() <= 2.0 ** -11
    assert np.abs(hi + lo - want).max() <= 2.0 ** -21
    inb = raw[32768:32768 + 65536].view(np.float64).reshape(64, 64, 2)
    assert np.abs(inb[..., 0] - np.cos(j)).max() < 1e-15 and np.abs(inb[..., 1] - np.sin(j)).max() < 1e-15
    rec = raw[98304:].reshape(MAX_POS // 64, 1536)
    ang = (64.0 * np.arange(MAX_POS // 64))[:, None] * f64[None, :]
    b32 = rec[:, :512].copy().view(np.float32).reshape(-1, 64, 2)
    b64 = rec[:, 512:].copy().view(np.float64).reshape(-1, 64, 2)
    # the argument itself is exact in fp64 up to one rounding (about 1e-10 at the largest angles)
    assert np.abs(b64[..., 0] - np.cos(ang)).max() < 1e-9 and np.abs(b64[..., 1] - np.sin(ang)).max() < 1e-9
    assert np.abs(b32[..., 0] - np.cos(ang)).max() < 1e-7 and np.abs(b32[..., 1] - np.sin(ang)).max() < 1e-7


ENC_CASES = [
    # name, batch, hkv, lens, starts, sub, G, page, sign
    ("2bit-groups-ragged", 2, 2, [300, 77], None, 4, 64, 0, False),
    ("1bit-onegroup", 1, 1, [515], None, 8, 0, 0, False),
    ("sign-groups-paged", 2, 1, [260, 130], None, 8, 64, 256, True),
    ("2bit-far-positions", 2, 1, [200, 64], [131072 - 256, 65536], 4, 64, 0, False),
]


@pytest.mark.parametrize("name,batch,hkv,lens,starts,sub,G,page,sign", ENC_CASES, ids=[c[0] for c in ENC_CASES])
def test_pre_rope_encode_matches_oracle(gpu_api, codebooks, magnitude_codebook, rope, name, batch, hkv, lens, starts,
                                        sub, G, page, sign):
    f, table = rope
    print(f"case {name} lens={lens} starts={starts} sub={sub} G={G} page={page} sign={sign}", flush=True)
    cb = magnitude_codebook if sign else codebooks[sub]
    seed = 900 + len(name)
    max_len = MAX_POS if starts else None
    k, v, hk, hv = run_gpu_encode(gpu_api, seed, batch, hkv, lens, sub, G, cb, page, starts=starts, sign=sign,
                                  rope_table=table, max_len=max_len)
    flips = 0
    for b in range(batch):
        s0 = starts[b] if starts else 0
        for h in range(hkv):
            fk, fv = hk.unit_dict(b, h, s0 + lens[b]), hv.unit_dict(b, h, s0 + lens[b])
            cut = lambda d: dict(codes=d["codes"][s0:], a=d["a"][s0:], b=d["b"][s0:], o=d["o"])
            flips += check_unit(k[b, h, :lens[b]], cut(fk), cb, G, start=s0, sign=sign, rope_inv_freq=f)
            flips += check_unit(v[b, h, :lens[b]], cut(fv), cb, G, start=s0, sign=sign)   # values: no embedding
    print(f"  near-tie code differences: {flips}", flush=True)


def test_pre_rope_append_with_frozen_means(gpu_api, codebooks, rope):
    f, table = rope
    cb = codebooks[4]
    lens0 = [192, 64]
    k0, v0, hk, hv = run_gpu_encode(gpu_api, 43, 2, 2, lens0, 4, 0, cb, max_len=256, rope_table=table)
    k1, v1, hk, hv = run_gpu_encode(gpu_api, 43, 2, 2, [3, 1], 4, 0, cb, starts=lens0, freeze=True,
                                    caches=(hk, hv), max_len=256, rope_table=table)
    for b, (s, n) in enumerate(zip(lens0, [3, 1])):
        for h in range(2):
            full = hk.unit_dict(b, h, s + n)
            got = dict(codes=full["codes"][s:], a=full["a"][s:], b=full["b"][s:], o=full["o"])
            check_unit(k1[b, h, :n], got, cb, 0, start=s, frozen=full["o"], rope_inv_freq=f)
            check_unit(k0[b, h, :s], hk.unit_dict(b, h, s), cb, 0, rope_inv_freq=f)


DEC_CASES = [
    # name, hq, hkv, lens, sub, G, page, splits, sign
    ("gqa4-2bit-groups", 8, 2, [777, 130], 4, 64, 0, 4, False),
    ("gqa4-2bit-onegroup", 4, 1, [1030, 1], 4, 0, 0, 0, False),
    ("mha-1bit", 2, 2, [333, 700], 8, 64, 0, 2, False),
    ("gqa2-1bit-paged", 4, 2, [900, 511], 8, 128, 256, 3, False),
    ("empty-and-short", 3, 1, [0, 65], 4, 64, 0, 2, False),
    ("gqa4-sign-groups", 4, 1, [600, 64], 8, 64, 0, 0, True),
    ("gqa8-two-launches", 8, 1, [300, 129], 4, 64, 0, 2, False),
    ("long-six-iterations-per-wave", 4, 1, [6000], 4, 64, 0, 2, False),   # more than one batch of four groups per wave
    ("long-onegroup-1bit", 2, 1, [5000], 8, 0, 0, 2, False),
]


def _build(seed, hkv, lens, sub, G, cb, page, sign, f):
    batch = len(lens)
    J = (2 if sign else 1) * (128 // sub)
    max_len = ((max(max(lens), 1) + 255) // 256) * 256
    bt = synth.shuffled_page_table(seed, batch, max_len // page) if page else None
    kc = helpers.HostCache("k", batch, hkv, J, max_len, G, page, bt, layout="legacy")
    vc = helpers.HostCache("v", batch, hkv, J, max_len, G, page, bt, layout="legacy")
    for b in range(batch):
        for h in range(hkv):
            if lens[b]:
                kc.put_unit(b, h, O.encode(synth.make_k(seed, b, h, lens[b]), cb, G, sign_format=sign, rope_inv_freq=f))
                vc.put_unit(b, h, O.encode(synth.make_v(seed, b, h, lens[b]), cb, G, sign_format=sign))
    return kc, vc, max_len


@pytest.mark.parametrize("name,hq,hkv,lens,sub,G,page,splits,sign", DEC_CASES, ids=[c[0] for c in DEC_CASES])
def test_pre_rope_decode_matches_oracle(gpu_api, codebooks, magnitude_codebook, rope, name, hq, hkv, lens, sub, G,
                                        page, splits, sign):
    import torch
    api = gpu_api
    f, table = rope
    print(f"case {name} lens={lens} sub={sub} G={G} page={page} splits={splits} sign={sign}", flush=True)
    cb = magnitude_codebook if sign else codebooks[sub]
    batch, r = len(lens), hq // hkv
    seed = 950 + len(name)
    scale = 1.0 / math.sqrt(128)
    kc, vc, max_len = _build(seed, hkv, lens, sub, G, cb, page, sign, f)
    q = synth.make_q(seed, batch, hq)
    shape = api.make_shape(sub, hq, hkv, max_len, G, page, sign_format=sign, rope_table=table)
    cbd = torch.from_numpy(cb.astype(np.float16)).cuda()
    out = api.nsn_decode_attention(shape, cbd, torch.from_numpy(q).cuda(), kc.to_device(api, shape),
                                   vc.to_device(api, shape), torch.tensor(lens, dtype=torch.int32).cuda(),
                                   max(lens), scale, splits)
    torch.cuda.synchronize()
    out = out.cpu().numpy().astype(np.float64)
    worst, moved = 0.0, 0.0
    for b in range(batch):
        if lens[b] == 0:
            assert np.all(out[b] == 0.0)
            continue
        for h in range(hkv):
            qh = q[b, h * r:(h + 1) * r].astype(np.float64)
            ku, vu = kc.unit_dict(b, h, lens[b]), vc.unit_dict(b, h, lens[b])
            ref = O.decode_attention(qh, ku, vu, cb, scale, G, sign_format=sign, rope_inv_freq=f)
            worst = max(worst, helpers.max_rel_err(out[b, h * r:(h + 1) * r], ref))
            moved = max(moved, helpers.max_rel_err(O.decode_attention(qh, ku, vu, cb, scale, G, sign_format=sign), ref))
    print(f"  max rel err {worst:.3e} (leaving the mean un-turned would give {moved:.3e})", flush=True)
    assert worst < TOL, worst


def test_pre_rope_generation_with_residual_and_flush(gpu_api, codebooks, rope):
    """The paper's decode loop with un-embedded keys: new tokens wait in the fp16 residual (embedded
    copies for attention, un-embedded copies for the encoder); a full residual is encoded as one
    64-token Shift group; attention turns the means of the coded groups in the kernel."""
    import torch
    api = gpu_api
    f, table = rope
    sub, B, Hq, Hkv, G, seed, steps = 4, 2, 8, 2, 64, 88, 70
    r, J, CAP = Hq // Hkv, 32, 64
    cb = codebooks[sub]
    prefill = [200, 64]
    max_len = 512
    shape = api.make_shape(sub, Hq, Hkv, max_len, G, 0, rope_table=table)
    cbd = torch.from_numpy(cb.astype(np.float16)).cuda()
    kc, vc = api.alloc_cache(shape, B), api.alloc_cache(shape, B)
    scale = 1.0 / math.sqrt(128)
    total = max(prefill) + steps
    xk = np.zeros((B, Hkv, total, 128), dtype=np.float16)      # keys before the embedding
    xk_rot = np.zeros_like(xk)                                  # and after it (fp16, as a model would hold them)
    xv = np.zeros_like(xk)
    for b in range(B):
        for h in range(Hkv):
            xk[b, h] = synth.make_k(seed, b, h, total)
            xk_rot[b, h] = O.rope(xk[b, h].astype(np.float64), np.arange(total), f).astype(np.float16)
            xv[b, h] = synth.make_v(seed, b, h, total)
    coded = [(n // G) * G for n in prefill]
    res_n = [n - c for n, c in zip(prefill, coded)]
    api.nsn_encode(shape, cbd, torch.from_numpy(xk[:, :, :max(coded)].copy()).cuda(),
                   torch.from_numpy(xv[:, :, :max(coded)].copy()).cuda(), torch.zeros(B, dtype=torch.int32).cuda(),
                   torch.tensor(coded, dtype=torch.int32).cuda(), kc, vc)
    k_res = torch.zeros((B, Hkv, CAP, 128), dtype=torch.float16).cuda()      # after the embedding: attention
    k_res_pre = torch.zeros_like(k_res)                                       # before it: the encoder's input
    v_res = torch.zeros_like(k_res)
    for b in range(B):
        k_res[b, :, :res_n[b]] = torch.from_numpy(xk_rot[b, :, coded[b]:prefill[b]]).cuda()
        k_res_pre[b, :, :res_n[b]] = torch.from_numpy(xk[b, :, coded[b]:prefill[b]]).cuda()
        v_res[b, :, :res_n[b]] = torch.from_numpy(xv[b, :, coded[b]:prefill[b]]).cuda()
    dec_ws = torch.zeros(api.nsn_workspace_bytes(shape, api.NSN_OP_DECODE, B), dtype=torch.uint8).cuda()

    def host_unit(dc, kind, b, h, length):
        codes = helpers.unpack_codes(dc.codes[b, h].cpu().numpy(), kind, J, "legacy")[:length]
        norms = dc.norms[b, h].cpu().numpy()[:length]
        return dict(codes=codes, a=norms[:, 0], b=norms[:, 1], o=dc.means[b, h].cpu().numpy()[:max(1, length // G)])

    worst, flushes = 0.0, 0
    pos = list(prefill)
    for step in range(steps):
        for b in range(B):
            k_res[b, :, res_n[b]] = torch.from_numpy(xk_rot[b, :, pos[b]]).cuda()
            k_res_pre[b, :, res_n[b]] = torch.from_numpy(xk[b, :, pos[b]]).cuda()
            v_res[b, :, res_n[b]] = torch.from_numpy(xv[b, :, pos[b]]).cuda()
            res_n[b] += 1
            pos[b] += 1
        q = synth.make_q(seed, B, Hq, step=step)
        out = api.nsn_decode_attention_residual(
            shape, cbd, torch.from_numpy(q).cuda(), kc, vc, torch.tensor(coded, dtype=torch.int32).cuda(),
            max(coded), k_res, v_res, torch.tensor(res_n, dtype=torch.int32).cuda(), scale, 0, workspace=dec_ws)
        torch.cuda.synchronize()
        if step % 9 == 0 or step == steps - 1 or max(res_n) == CAP:
            out_h = out.cpu().numpy().astype(np.float64)
            for b in range(B):
                for h in range(Hkv):
                    gk, gv = host_unit(kc, "k", b, h, coded[b]), host_unit(vc, "v", b, h, coded[b])
                    ref = O.decode_attention_residual(
                        q[b, h * r:(h + 1) * r].astype(np.float64), gk, gv, xk_rot[b, h, coded[b]:pos[b]],
                        xv[b, h, coded[b]:pos[b]], cb, scale, G, rope_inv_freq=f)
                    worst = max(worst, helpers.max_rel_err(out_h[b, h * r:(h + 1) * r], ref))
        full = [n == CAP for n in res_n]
        if any(full):
            n_new = [CAP if fl else 0 for fl in full]
            api.nsn_encode(shape, cbd, k_res_pre, v_res, torch.tensor(coded, dtype=torch.int32).cuda(),
                           torch.tensor(n_new, dtype=torch.int32).cuda(), kc, vc)
            torch.cuda.synchronize()
            for b in range(B):
                if not full[b]:
                    continue
                flushes += 1
                for h in range(Hkv):
                    gk = host_unit(kc, "k", b, h, coded[b] + CAP)
                    grp = coded[b] // G
                    check_unit(xk[b, h, coded[b]:coded[b] + CAP],
                               dict(codes=gk["codes"][coded[b]:], a=gk["a"][coded[b]:], b=gk["b"][coded[b]:],
                                    o=gk["o"][:grp + 1]), cb, G, start=coded[b], rope_inv_freq=f)
                coded[b] += CAP
                res_n[b] = 0
    print(f"  {flushes} flushes, worst decode max rel err {worst:.3e}", flush=True)
    assert flushes >= 2
    assert worst < TOL, worst
