"""Ragged prefill + paged layout + decode steps that append one token per sequence per step
(Mistral-7B shape: 32 query heads over 8 kv heads; lengths uniform in [512, 16384]; 256-token pages
in shuffled physical order; Shift mean over each sequence's prefill, frozen for appended tokens).
Runs at 1-bit and 2-bit over the whole seeded 32-sequence batch; the oracle re-computes sampled
(sequence, head) units: the longest sequence, the shortest one and the last one."""
import math

import numpy as np
import pytest

from oracle import nsn_oracle as O
from paper_2505_18231_amd import synth
from tests import helpers
from tests.test_gpu_encode import check_unit

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("sub", [8, 4])
def test_ragged_paged_prefill_then_append_steps(gpu_api, codebooks, sub):
    import torch
    api = gpu_api
    cfg = synth.CONFIGS["C4"]
    cb = codebooks[sub]
    B, Hq, Hkv, page, steps, seed = cfg["batch"], cfg["n_q_heads"], cfg["n_kv_heads"], cfg["page_size"], cfg["append_steps"], cfg["seed"]
    r = Hq // Hkv
    J = 128 // sub
    lens = synth.ragged_lengths(seed, cfg["batch"], cfg["len_lo"], cfg["len_hi"])[:B].tolist()
    max_len = ((max(lens) + steps + page - 1) // page) * page
    n_pages_seq = max_len // page
    bt = synth.shuffled_page_table(seed, B, n_pages_seq)
    print(f"case sub={sub} lens={lens} max_len={max_len}", flush=True)
    shape = api.make_shape(sub, Hq, Hkv, max_len, 0, page)
    btd = torch.from_numpy(bt).cuda()
    kc = api.alloc_cache(shape, B, block_table=btd)
    vc = api.alloc_cache(shape, B, block_table=btd)
    cbd = torch.from_numpy(cb.astype(np.float16)).cuda()
    scale = 1.0 / math.sqrt(128)
    sample = sorted({(int(np.argmax(lens)), 0), (int(np.argmin(lens)), Hkv - 1), (B - 1, Hkv - 1)})

    # ragged prefill
    max_new = max(lens)
    k = np.zeros((B, Hkv, max_new, 128), dtype=np.float16)
    v = np.zeros_like(k)
    for b in range(B):
        for h in range(Hkv):
            k[b, h, :lens[b]] = synth.make_k(seed, b, h, lens[b])
            v[b, h, :lens[b]] = synth.make_v(seed, b, h, lens[b])
    lens_d = torch.tensor(lens, dtype=torch.int32).cuda()
    api.nsn_encode(shape, cbd, torch.from_numpy(k).cuda(), torch.from_numpy(v).cuda(),
                   torch.zeros(B, dtype=torch.int32).cuda(), lens_d, kc, vc)

    # oracle caches of the sampled units (prefill part)
    ok = {u: O.encode(k[u[0], u[1], :lens[u[0]]], cb, 0) for u in sample}
    ov = {u: O.encode(v[u[0], u[1], :lens[u[0]]], cb, 0) for u in sample}
    dec_ws = torch.zeros(api.nsn_workspace_bytes(shape, api.NSN_OP_DECODE, B), dtype=torch.uint8).cuda()

    def host_unit(dc, kind, b, h, length):
        codes = np.concatenate([helpers.unpack_codes(dc.codes[bt[b, p], h].cpu().numpy(), kind, J)
                                for p in range(n_pages_seq)])[:length]
        norms = np.concatenate([dc.norms[bt[b, p], h].cpu().numpy() for p in range(n_pages_seq)])[:length]
        return dict(codes=codes, a=norms[:, 0], b=norms[:, 1], o=dc.means[b, h].cpu().numpy())

    cur = list(lens)
    worst = 0.0
    for step in range(steps):
        # append one new token per sequence, encoded with the frozen prefill mean
        k1 = np.zeros((B, Hkv, 1, 128), dtype=np.float16)
        v1 = np.zeros_like(k1)
        for b in range(B):
            for h in range(Hkv):
                k1[b, h, 0] = synth.make_k(seed, b, h, 1, start=cur[b])[0]
                v1[b, h, 0] = synth.make_v(seed, b, h, 1, start=cur[b])[0]
        api.nsn_encode(shape, cbd, torch.from_numpy(k1).cuda(), torch.from_numpy(v1).cuda(),
                       torch.tensor(cur, dtype=torch.int32).cuda(), torch.ones(B, dtype=torch.int32).cuda(),
                       kc, vc, freeze_means=True)
        for u in sample:
            ek = O.encode(k1[u[0], u[1]], cb, 0, start=cur[u[0]], frozen_o=ok[u]["o"])
            ev = O.encode(v1[u[0], u[1]], cb, 0, start=cur[u[0]], frozen_o=ov[u]["o"])
            for key in ("codes", "a", "b"):
                ok[u][key] = np.concatenate([ok[u][key], ek[key]])
                ov[u][key] = np.concatenate([ov[u][key], ev[key]])
        cur = [c + 1 for c in cur]
        q = synth.make_q(seed, B, Hq, step=step)
        out = api.nsn_decode_attention(shape, cbd, torch.from_numpy(q).cuda(), kc, vc,
                                       torch.tensor(cur, dtype=torch.int32).cuda(), max(cur), scale, 0,
                                       workspace=dec_ws)
        torch.cuda.synchronize()
        if step in (0, steps - 1):
            out_h = out.cpu().numpy().astype(np.float64)
            for (b, h) in sample:
                gk, gv = host_unit(kc, "k", b, h, cur[b]), host_unit(vc, "v", b, h, cur[b])
                # the device cache equals the oracle's (codes bit-exact outside ties, a within one ulp)
                n_app = step + 1
                xk = np.concatenate([k[b, h, :lens[b]]] + [synth.make_k(seed, b, h, 1, start=lens[b] + i) for i in range(n_app)])
                tail = slice(lens[b], cur[b])
                check_unit(xk[tail], dict(codes=gk["codes"][tail], a=gk["a"][tail], b=gk["b"][tail], o=gk["o"]),
                           cb, 0, start=lens[b], frozen=gk["o"])
                if step == 0:
                    check_unit(xk[:lens[b]], dict(codes=gk["codes"][:lens[b]], a=gk["a"][:lens[b]],
                                                  b=gk["b"][:lens[b]], o=gk["o"]), cb, 0)
                ref = O.decode_attention(q[b, h * r:(h + 1) * r].astype(np.float64), gk, gv, cb, scale, 0)
                err = helpers.max_rel_err(out_h[b, h * r:(h + 1) * r], ref)
                # and against the oracle's own cache (differs at most in near-tie codes)
                ref2 = O.decode_attention(q[b, h * r:(h + 1) * r].astype(np.float64), ok[(b, h)], ov[(b, h)], cb, scale, 0)
                err2 = helpers.max_rel_err(out_h[b, h * r:(h + 1) * r], ref2)
                print(f"  step {step} unit (b={b}, h={h}) len={cur[b]}: decode max rel err {err:.3e} "
                      f"(vs oracle-encoded cache {err2:.3e})", flush=True)
                worst = max(worst, err)
                assert err2 < 5e-3
    assert worst < 2e-3, worst
