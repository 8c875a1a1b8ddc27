"""GPU parity of nsn_decode_attention_residual (Sec. 3.2 "Residual": the most recent tokens stay
fp16 and join the softmax of the coded tokens), and of the generation policy built on it:
tokens collect in the residual, and when 64 have arrived they are encoded as one Shift group
(group size 64, the paper's setting) by nsn_encode reading the residual buffers directly.
Tolerance: 2e-3 max relative error per output row, as for the coded-only decode."""
import math

import numpy as np
import pytest

from oracle import nsn_oracle as O
from paper_2505_18231_amd import synth
from tests import helpers
from tests.test_gpu_encode import check_unit

pytestmark = pytest.mark.gpu
TOL = 2e-3
CAP = 64

CASES = [
    # name, hq, hkv, coded lens, residual lens, sub, G, page, splits
    ("gqa4-2bit", 8, 2, [640, 128, 0, 1024], [37, 64, 5, 0], 4, 64, 0, 0),
    ("gqa4-1bit", 4, 1, [256, 0, 64], [1, 64, 63], 8, 64, 0, 3),
    ("mha-2bit", 2, 2, [320, 64], [17, 33], 4, 64, 0, 2),
    ("gqa2-1bit-paged", 4, 2, [512, 768], [64, 2], 8, 64, 256, 0),
    ("gqa3-2bit-onegroup", 3, 1, [500, 77], [20, 64], 4, 0, 0, 4),   # 3 heads run in the 4-head kernel
    ("residual-only", 4, 1, [0, 0], [64, 9], 4, 64, 0, 0),
    ("nothing-at-all", 4, 1, [0, 192], [0, 0], 8, 64, 0, 0),
    ("gqa8-two-launches", 16, 2, [384, 64], [33, 64], 4, 64, 0, 0),   # 8 query heads per kv head
    ("gqa5-two-launches", 5, 1, [130], [7], 8, 0, 0, 2),              # 4 + 1
    ("long-eleven-waves", 4, 1, [4608, 64], [64, 3], 4, 64, 0, 1),    # 4096+ token split: 11 main waves + the residual wave
    # 128 units, automatic splitting: the persistent instance; the segment with a unit's last group takes the
    # residual, also for units without coded tokens
    ("flat-ragged-2bit", 32, 8, [0, 1, 64, 65, 130, 300, 17, 256, 511, 77, 128, 5, 200, 333, 90, 400],
     [3, 64, 0, 17, 33, 64, 1, 0, 20, 5, 64, 63, 2, 48, 0, 9], 4, 64, 0, 0),
    ("flat-paged-1bit-gqa8", 64, 8, [700, 0, 64, 65, 130, 900, 17, 256, 511, 77, 128, 5, 200, 333, 90, 0],
     [64, 0, 0, 17, 33, 64, 1, 0, 20, 5, 64, 63, 2, 48, 0, 9], 8, 0, 256, 0),
]


@pytest.mark.parametrize("name,hq,hkv,lens,rlens,sub,G,page,splits", CASES, ids=[c[0] for c in CASES])
def test_residual_decode_matches_oracle(gpu_api, codebooks, name, hq, hkv, lens, rlens, sub, G, page, splits):
    import torch
    api = gpu_api
    print(f"case {name} lens={lens} residual={rlens} sub={sub} G={G} page={page} splits={splits}", flush=True)
    cb = codebooks[sub]
    batch, r, J = len(lens), hq // hkv, 128 // sub
    seed = 300 + len(name)
    scale = 1.0 / math.sqrt(128)
    max_len = ((max(max(lens), 1) + 255) // 256) * 256
    bt = synth.shuffled_page_table(seed, batch, max_len // page) if page else None
    kc = helpers.HostCache("k", batch, hkv, J, max_len, G, page, bt)
    vc = helpers.HostCache("v", batch, hkv, J, max_len, G, page, bt)
    k_res = np.zeros((batch, hkv, CAP, 128), dtype=np.float16)
    v_res = np.zeros_like(k_res)
    # rows past the valid count hold values that would poison the result if they were read
    k_res[:] = np.float16(np.inf)
    v_res[:] = np.float16(np.nan)
    for b in range(batch):
        for h in range(hkv):
            if lens[b]:
                kc.put_unit(b, h, O.encode(synth.make_k(seed, b, h, lens[b]), cb, G))
                vc.put_unit(b, h, O.encode(synth.make_v(seed, b, h, lens[b]), cb, G))
            k_res[b, h, :rlens[b]] = synth.make_k(seed, b, h, rlens[b], start=lens[b])
            v_res[b, h, :rlens[b]] = synth.make_v(seed, b, h, rlens[b], start=lens[b])
    q = synth.make_q(seed, batch, hq)
    shape = api.make_shape(sub, hq, hkv, max_len, G, page)
    cbd = torch.from_numpy(cb.astype(np.float16)).cuda()
    out = api.nsn_decode_attention_residual(
        shape, cbd, torch.from_numpy(q).cuda(), kc.to_device(api, shape), vc.to_device(api, shape),
        torch.tensor(lens, dtype=torch.int32).cuda(), max(lens), torch.from_numpy(k_res).cuda(),
        torch.from_numpy(v_res).cuda(), torch.tensor(rlens, dtype=torch.int32).cuda(), scale, splits)
    torch.cuda.synchronize()
    out = out.cpu().numpy().astype(np.float64)
    worst = 0.0
    for b in range(batch):
        if lens[b] + rlens[b] == 0:
            assert np.all(out[b] == 0.0)
            continue
        for h in range(hkv):
            ref = O.decode_attention_residual(
                q[b, h * r:(h + 1) * r].astype(np.float64), kc.unit_dict(b, h, lens[b]), vc.unit_dict(b, h, lens[b]),
                k_res[b, h, :rlens[b]], v_res[b, h, :rlens[b]], cb, scale, G)
            worst = max(worst, helpers.max_rel_err(out[b, h * r:(h + 1) * r], ref))
    print(f"  max rel err {worst:.3e}", flush=True)
    assert worst < TOL, worst


def test_residual_with_no_rows_equals_plain_decode(gpu_api, codebooks):
    import torch
    api = gpu_api
    cb = codebooks[4]
    lens = [700, 130]
    from tests.test_gpu_decode import build_case
    kc, vc, q, max_len = build_case(11, 2, 8, 2, lens, 4, 64, cb)
    shape = api.make_shape(4, 8, 2, max_len, 64, 0)
    cbd = torch.from_numpy(cb.astype(np.float16)).cuda()
    dk, dv = kc.to_device(api, shape), vc.to_device(api, shape)
    lens_d = torch.tensor(lens, dtype=torch.int32).cuda()
    qd = torch.from_numpy(q).cuda()
    scale = 1.0 / math.sqrt(128)
    plain = api.nsn_decode_attention(shape, cbd, qd, dk, dv, lens_d, max(lens), scale, 3)
    empty = torch.zeros((2, 2, CAP, 128), dtype=torch.float16).cuda()
    with_res = api.nsn_decode_attention_residual(shape, cbd, qd, dk, dv, lens_d, max(lens), empty, empty,
                                                 torch.zeros(2, dtype=torch.int32).cuda(), scale, 3)
    torch.cuda.synchronize()
    assert torch.equal(plain, with_res)


@pytest.mark.parametrize("sub", [4, 8])
def test_generation_with_residual_and_group_flush(gpu_api, codebooks, sub):
    """Prefill in whole 64-token groups, the remainder in the residual; every step appends one
    token to the residual, attends, and flushes a full residual into the coded cache."""
    import torch
    api = gpu_api
    cb = codebooks[sub]
    B, Hq, Hkv, G, seed, steps = 3, 8, 2, 64, 77, 70
    r, J = Hq // Hkv, 128 // sub
    prefill = [200, 64, 37]
    max_len = 512
    shape = api.make_shape(sub, Hq, Hkv, max_len, G, 0)
    cbd = torch.from_numpy(cb.astype(np.float16)).cuda()
    kc, vc = api.alloc_cache(shape, B), api.alloc_cache(shape, B)
    scale = 1.0 / math.sqrt(128)
    total = max(prefill) + steps
    xk = np.zeros((B, Hkv, total, 128), dtype=np.float16)
    xv = np.zeros_like(xk)
    for b in range(B):
        for h in range(Hkv):
            xk[b, h] = synth.make_k(seed, b, h, total)
            xv[b, h] = synth.make_v(seed, b, h, total)

    coded = [(n // G) * G for n in prefill]
    res_n = [n - c for n, c in zip(prefill, coded)]
    k_in = torch.from_numpy(xk[:, :, :max(coded)].copy()).cuda()
    v_in = torch.from_numpy(xv[:, :, :max(coded)].copy()).cuda()
    api.nsn_encode(shape, cbd, k_in, v_in, torch.zeros(B, dtype=torch.int32).cuda(),
                   torch.tensor(coded, dtype=torch.int32).cuda(), kc, vc)
    k_res = torch.zeros((B, Hkv, CAP, 128), dtype=torch.float16).cuda()
    v_res = torch.zeros_like(k_res)
    for b in range(B):
        k_res[b, :, :res_n[b]] = torch.from_numpy(xk[b, :, coded[b]:prefill[b]]).cuda()
        v_res[b, :, :res_n[b]] = torch.from_numpy(xv[b, :, coded[b]:prefill[b]]).cuda()
    dec_ws = torch.zeros(api.nsn_workspace_bytes(shape, api.NSN_OP_DECODE, B), dtype=torch.uint8).cuda()

    def host_unit(dc, kind, b, h, length):
        codes = helpers.unpack_codes(dc.codes[b, h].cpu().numpy(), kind, J)[:length]
        norms = dc.norms[b, h].cpu().numpy()[:length]
        return dict(codes=codes, a=norms[:, 0], b=norms[:, 1], o=dc.means[b, h].cpu().numpy()[:max(1, length // G)])

    worst, flushes = 0.0, 0
    pos = list(prefill)
    for step in range(steps):
        for b in range(B):  # the new token of every sequence goes to the residual
            k_res[b, :, res_n[b]] = torch.from_numpy(xk[b, :, pos[b]]).cuda()
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
                        q[b, h * r:(h + 1) * r].astype(np.float64), gk, gv, xk[b, h, coded[b]:pos[b]],
                        xv[b, h, coded[b]:pos[b]], cb, scale, G)
                    worst = max(worst, helpers.max_rel_err(out_h[b, h * r:(h + 1) * r], ref))
        full = [n == CAP for n in res_n]
        if any(full):  # a full residual becomes one coded Shift group, straight from its buffer
            n_new = [CAP if f else 0 for f in full]
            api.nsn_encode(shape, cbd, k_res, v_res, torch.tensor(coded, dtype=torch.int32).cuda(),
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
                                    o=gk["o"][grp:grp + 1]), cb, G)
                coded[b] += CAP
                res_n[b] = 0
    print(f"  sub={sub}: {flushes} flushes, worst decode max rel err {worst:.3e}", flush=True)
    assert flushes >= 3
    assert worst < TOL, worst
