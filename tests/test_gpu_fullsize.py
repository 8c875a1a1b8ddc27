"""Full-size GPU parity in the launch configuration bench.py times (Llama-3-8B shape, 2-bit,
batch 8 x 8192 tokens, 32 query heads over 8 kv heads, one Shift group per sequence, automatic
split count), plus the long-context 1-bit shape (131072 tokens, batch 1) and the large-batch
multi-head shape (64 sequences x 32768 tokens, 32 heads).

The GPU encodes and decodes the whole batch; the oracle re-computes a sample of (sequence, kv-head)
units: the encoder's two-stage check on those units, and decode attention on the very cache bytes
the GPU produced (so the decode comparison is exact up to arithmetic, not up to code ties)."""
import math

import numpy as np
import pytest

from oracle import nsn_oracle as O
from paper_2505_18231_amd import synth
from tests import helpers
from tests.test_gpu_encode import check_unit

pytestmark = pytest.mark.gpu


def check_unit_sampled(x16, got, cb, n_tokens, seed):
    """Long sequences (one Shift group): stage A on every token, stage B on a seeded token sample,
    conditioned on the device's stored b and o (tokens are independent once b and o are fixed)."""
    b_ref, o_ref = O.shift_stats(x16, 0)
    assert np.array_equal(b_ref.view(np.uint16), got["b"].view(np.uint16)), "first-Normalize scale"
    assert np.array_equal(o_ref.view(np.uint16), got["o"][:1].view(np.uint16)), "means"
    idx = np.sort(np.random.default_rng(seed).choice(x16.shape[0], size=n_tokens, replace=False))
    part = dict(codes=got["codes"][idx], a=got["a"][idx], b=got["b"][idx], o=got["o"][:1])
    return check_unit(x16[idx], part, cb, 0, frozen=got["o"][:1])


def _run(api, cfg_name, cb, sample_units, G=0, token_sample=None, batch=None, device_fill=False):
    import torch
    cfg = synth.CONFIGS[cfg_name]
    B, Hq, Hkv, L, sub, seed = (batch or cfg["batch"], cfg["n_q_heads"], cfg["n_kv_heads"], cfg["length"],
                                cfg["sub_dim"], cfg["seed"])
    J = 128 // sub
    r = Hq // Hkv
    scale = 1.0 / math.sqrt(128)
    print(f"case {cfg_name} B={B} Hq={Hq} Hkv={Hkv} L={L} sub={sub}", flush=True)
    shape = api.make_shape(sub, Hq, Hkv, L, G)
    kc, vc = api.alloc_cache(shape, B), api.alloc_cache(shape, B)
    cbd = torch.from_numpy(cb.astype(np.float16)).cuda()
    zeros = torch.zeros(B, dtype=torch.int32).cuda()
    full = torch.full((B,), L, dtype=torch.int32).cuda()
    # encode one sequence at a time (bounds host and device staging memory)
    k_units, v_units = {}, {}
    gen = torch.Generator(device="cuda").manual_seed(seed)
    for b in range(B):
        if device_fill:
            # units the oracle does not re-compute are drawn on the device (same recipe: per-channel scale
            # and bias for keys, N(0,1) values); the sampled units below come from the host generator
            st = [synth.channel_stats(seed, b, h, per_seq=cfg.get("per_seq", False)) for h in range(Hkv)]
            sc = torch.tensor(np.stack([s_[0] for s_ in st]), dtype=torch.float32, device="cuda")[:, None, :]
            bi = torch.tensor(np.stack([s_[1] for s_ in st]), dtype=torch.float32, device="cuda")[:, None, :]
            kd_ = (torch.randn((Hkv, L, 128), generator=gen, device="cuda") * sc + bi).half()[None]
            vd_ = torch.randn((Hkv, L, 128), generator=gen, device="cuda").half()[None]
            for h in range(Hkv):
                if (b, h) in sample_units:
                    k_units[(b, h)] = synth.make_k(seed, b, h, L, per_seq=cfg.get("per_seq", False))
                    v_units[(b, h)] = synth.make_v(seed, b, h, L)
                    kd_[0, h] = torch.from_numpy(k_units[(b, h)]).cuda()
                    vd_[0, h] = torch.from_numpy(v_units[(b, h)]).cuda()
        else:
            k = np.empty((1, Hkv, L, 128), dtype=np.float16)
            v = np.empty_like(k)
            for h in range(Hkv):
                k[0, h] = synth.make_k(seed, b, h, L, per_seq=cfg.get("per_seq", False))
                v[0, h] = synth.make_v(seed, b, h, L)
                if (b, h) in sample_units:
                    k_units[(b, h)], v_units[(b, h)] = k[0, h].copy(), v[0, h].copy()
            kd_, vd_ = torch.from_numpy(k).cuda(), torch.from_numpy(v).cuda()
        sub_k = api.CodedCache(kc.codes[b:b + 1], kc.norms[b:b + 1], kc.means[b:b + 1], None)
        sub_v = api.CodedCache(vc.codes[b:b + 1], vc.norms[b:b + 1], vc.means[b:b + 1], None)
        api.nsn_encode(shape, cbd, kd_, vd_, zeros[:1], full[:1], sub_k, sub_v)
        if b % 8 == 7:
            torch.cuda.synchronize()
            print(f"  encoded sequences 0..{b}", flush=True)
    q = synth.make_q(seed, B, Hq)
    out = api.nsn_decode_attention(shape, cbd, torch.from_numpy(q).cuda(), kc, vc, full, L, scale, 0)
    torch.cuda.synchronize()
    out = out.cpu().numpy().astype(np.float64)
    worst = 0.0
    for (b, h) in sample_units:
        kd = dict(codes=helpers.unpack_codes(kc.codes[b, h].cpu().numpy(), "k", J)[:L],
                  a=kc.norms[b, h, :L, 0].cpu().numpy(), b=kc.norms[b, h, :L, 1].cpu().numpy(),
                  o=kc.means[b, h].cpu().numpy())
        vd = dict(codes=helpers.unpack_codes(vc.codes[b, h].cpu().numpy(), "v", J)[:L],
                  a=vc.norms[b, h, :L, 0].cpu().numpy(), b=vc.norms[b, h, :L, 1].cpu().numpy(),
                  o=vc.means[b, h].cpu().numpy())
        if token_sample:
            flips = (check_unit_sampled(k_units[(b, h)], kd, cb, token_sample, 1) +
                     check_unit_sampled(v_units[(b, h)], vd, cb, token_sample, 2))
        else:
            flips = check_unit(k_units[(b, h)], kd, cb, G) + check_unit(v_units[(b, h)], vd, cb, G)
        ref = O.decode_attention(q[b, h * r:(h + 1) * r].astype(np.float64), kd, vd, cb, scale, G)
        err = helpers.max_rel_err(out[b, h * r:(h + 1) * r], ref)
        print(f"  unit (b={b}, h={h}): near-tie code differences {flips}, decode max rel err {err:.3e}", flush=True)
        worst = max(worst, err)
    assert worst < 2e-3, worst
    # properties that hold at any size: finite outputs, and |out| bounded by the largest value token norm
    assert np.isfinite(out).all()


def test_llama3_8b_2bit_full_shape(gpu_api, codebooks):
    _run(gpu_api, "C1", codebooks[4], [(0, 0), (3, 5), (7, 7)])


def test_long_context_1bit_full_shape(gpu_api, codebooks):
    _run(gpu_api, "C2", codebooks[8], [(0, 2)], token_sample=4096)


def test_mha_large_batch_full_shape(gpu_api, codebooks):
    # Llama-2-7B shape (32 kv heads = 32 query heads, 32768 tokens, 2-bit, per-sequence channel biases),
    # all 64 sequences in one decode launch; the oracle re-computes five (sequence, head) units, the
    # last sequence's last head among them
    _run(gpu_api, "C3", codebooks[4], [(0, 0), (1, 31), (31, 7), (40, 16), (63, 31)], token_sample=2048,
         device_fill=True)


def test_llama3_8b_shape_in_the_papers_own_configuration(gpu_api):
    """Everything the paper's pipeline has, at the benchmark's size: sign + index 2-bit codes with a
    magnitude codebook, 64-token Shift groups, keys normalised before the rotary embedding (the mean is
    turned inside the attention kernel), 4-bit side information, codebook entries on 16 levels, and a
    partly filled fp16 residual in the softmax.  The oracle re-computes three (sequence, head) units."""
    import torch
    from tests.test_gpu_double_quant import _check_unit
    api = gpu_api
    cfg = synth.CONFIGS["C1"]
    B, Hq, Hkv, L, seed = cfg["batch"], cfg["n_q_heads"], cfg["n_kv_heads"], cfg["length"], cfg["seed"]
    G, J, r, RES = 64, 32, Hq // Hkv, 64
    scale = 1.0 / math.sqrt(128)
    sample_units = [(0, 0), (3, 5), (7, 7)]
    x = np.abs(synth.codebook_samples(4242, 1 << 13, 8).astype(np.float64))
    cb, _, _ = O.build_codebook(x, 256, 5)
    cb, _, _, _ = O.quantize_codebook_4bit(cb)
    f = synth.rope_inv_freq(500000.0)
    table = api.nsn_build_rope_table(f, L + RES)
    shape = api.make_shape(8, Hq, Hkv, L + RES, G, sign_format=True, rope_table=table, side_bits=4)
    kc, vc = api.alloc_cache(shape, B), api.alloc_cache(shape, B)
    cbd = torch.from_numpy(cb.astype(np.float16)).cuda()
    zeros = torch.zeros(B, dtype=torch.int32).cuda()
    full = torch.full((B,), L, dtype=torch.int32).cuda()
    k_units, v_units = {}, {}
    res_rows = [37, 64, 1, 0, 12, 63, 5, 20]
    k_res = np.zeros((B, Hkv, RES, 128), dtype=np.float16)
    v_res = np.zeros_like(k_res)
    for b in range(B):
        k = np.empty((1, Hkv, L, 128), dtype=np.float16)
        v = np.empty_like(k)
        for h in range(Hkv):
            k[0, h] = synth.make_k(seed, b, h, L)
            v[0, h] = synth.make_v(seed, b, h, L)
            # residual keys are the embedded ones, as attention uses them
            k_res[b, h, :res_rows[b]] = O.rope(synth.make_k(seed, b, h, res_rows[b], start=L).astype(np.float64),
                                               L + np.arange(res_rows[b]), f).astype(np.float16)
            v_res[b, h, :res_rows[b]] = synth.make_v(seed, b, h, res_rows[b], start=L)
            if (b, h) in sample_units:
                k_units[(b, h)], v_units[(b, h)] = k[0, h].copy(), v[0, h].copy()
        sub_k = api.CodedCache(kc.codes[b:b + 1], kc.norms[b:b + 1], kc.means[b:b + 1], None)
        sub_v = api.CodedCache(vc.codes[b:b + 1], vc.norms[b:b + 1], vc.means[b:b + 1], None)
        api.nsn_encode(shape, cbd, torch.from_numpy(k).cuda(), torch.from_numpy(v).cuda(), zeros[:1], full[:1],
                       sub_k, sub_v)
    q = synth.make_q(seed, B, Hq)
    out = api.nsn_decode_attention_residual(shape, cbd, torch.from_numpy(q).cuda(), kc, vc, full, L,
                                            torch.from_numpy(k_res).cuda(), torch.from_numpy(v_res).cuda(),
                                            torch.tensor(res_rows, dtype=torch.int32).cuda(), scale, 0)
    torch.cuda.synchronize()
    out = out.cpu().numpy().astype(np.float64)
    hk = helpers.HostCacheDQ("k", B, Hkv, J, L + RES, G, layout="legacy")
    hv = helpers.HostCacheDQ("v", B, Hkv, J, L + RES, G, layout="legacy")
    hk.from_device(kc)
    hv.from_device(vc)
    worst = 0.0
    for (b, h) in sample_units:
        kd, vd = hk.unit_dict(b, h, L), hv.unit_dict(b, h, L)
        flips = (_check_unit(k_units[(b, h)], kd, cb, G, True, rope_inv_freq=f) +
                 _check_unit(v_units[(b, h)], vd, cb, G, True))
        ref = O.decode_attention_residual(q[b, h * r:(h + 1) * r].astype(np.float64), kd, vd,
                                          k_res[b, h, :res_rows[b]], v_res[b, h, :res_rows[b]], cb, scale, G,
                                          sign_format=True, rope_inv_freq=f)
        err = helpers.max_rel_err(out[b, h * r:(h + 1) * r], ref)
        print(f"  unit (b={b}, h={h}): near-tie code differences {flips}, decode max rel err {err:.3e}", flush=True)
        worst = max(worst, err)
    assert worst < 2e-3, worst
    assert np.isfinite(out).all()
