"""The library only enqueues kernels on the caller's stream (no allocation, no memset, no host
synchronisation in nsn_encode / nsn_decode_attention), so a decode step can be captured in a HIP
graph.  Replays must reproduce the eager results bit for bit (no floating-point atomics), with
eager work and synchronisations between the replays."""
import math

import numpy as np
import pytest

from paper_2505_18231_amd import synth

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("sub", [4, 8])
def test_decode_step_replays_bit_identically(gpu_api, codebooks, sub):
    import torch
    api = gpu_api
    B, Hq, Hkv, L, G = 2, 8, 2, 700, 0
    max_len = 768
    cb = torch.from_numpy(codebooks[sub].astype(np.float16)).cuda()
    shape = api.make_shape(sub, Hq, Hkv, max_len, G)
    kc, vc = api.alloc_cache(shape, B), api.alloc_cache(shape, B)
    k, v = synth.make_kv(61, B, Hkv, L)
    api.nsn_encode(shape, cb, torch.from_numpy(k).cuda(), torch.from_numpy(v).cuda(),
                   torch.zeros(B, dtype=torch.int32).cuda(), torch.full((B,), L, dtype=torch.int32).cuda(), kc, vc)
    scale = 1.0 / math.sqrt(128)
    # static buffers of the captured step
    k_new = torch.zeros((B, Hkv, 1, 128), dtype=torch.float16).cuda()
    v_new = torch.zeros_like(k_new)
    q = torch.zeros((B, Hq, 128), dtype=torch.float16).cuda()
    pos = torch.full((B,), L, dtype=torch.int32).cuda()
    one = torch.ones(B, dtype=torch.int32).cuda()
    lens = torch.full((B,), L + 1, dtype=torch.int32).cuda()
    out = torch.zeros((B, Hq, 128), dtype=torch.float32).cuda()
    enc_ws = torch.zeros(max(1, api.nsn_workspace_bytes(shape, api.NSN_OP_ENCODE, B, 1)), dtype=torch.uint8).cuda()
    dec_ws = torch.zeros(max(1, api.nsn_workspace_bytes(shape, api.NSN_OP_DECODE, B)), dtype=torch.uint8).cuda()

    def step():
        api.nsn_encode(shape, cb, k_new, v_new, pos, one, kc, vc, freeze_means=True, workspace=enc_ws)
        api.nsn_decode_attention(shape, cb, q, kc, vc, lens, L + 1, scale, 0, out=out, workspace=dec_ws)

    def set_inputs(i):
        k_new.copy_(torch.from_numpy(np.stack([[synth.make_k(61, b, h, 1, start=L + i) for h in range(Hkv)]
                                               for b in range(B)])))
        v_new.copy_(torch.from_numpy(np.stack([[synth.make_v(61, b, h, 1, start=L + i) for h in range(Hkv)]
                                               for b in range(B)])))
        q.copy_(torch.from_numpy(synth.make_q(61, B, Hq, step=i)))

    eager = []
    for i in range(3):
        set_inputs(i)
        step()
        torch.cuda.synchronize()
        eager.append(out.clone())

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()  # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for rep in range(2):
        for i in range(3):
            set_inputs(i)
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(out, eager[i]), f"replay {rep}/{i} differs from the eager result"
            # eager work between replays
            scratch = (out * 2).sum().item()
            assert np.isfinite(scratch)


def test_residual_step_and_flush_replay_bit_identically(gpu_api, codebooks):
    """The residual form of the step (nine-wave launch) and the 64-token flush encode, captured as two
    graphs and replayed against their eager results."""
    import torch
    api = gpu_api
    sub, B, Hq, Hkv, L, G = 4, 2, 8, 2, 640, 64
    cb = torch.from_numpy(codebooks[sub].astype(np.float16)).cuda()
    shape = api.make_shape(sub, Hq, Hkv, 768, G)
    kc, vc = api.alloc_cache(shape, B), api.alloc_cache(shape, B)
    k, v = synth.make_kv(62, B, Hkv, L + 64)
    kd, vd = torch.from_numpy(k).cuda(), torch.from_numpy(v).cuda()
    coded = torch.full((B,), L, dtype=torch.int32).cuda()
    api.nsn_encode(shape, cb, kd[:, :, :L].contiguous(), vd[:, :, :L].contiguous(),
                   torch.zeros(B, dtype=torch.int32).cuda(), coded, kc, vc)
    scale = 1.0 / math.sqrt(128)
    k_res, v_res = kd[:, :, L:].contiguous(), vd[:, :, L:].contiguous()
    res_len = torch.zeros(B, dtype=torch.int32).cuda()
    full = torch.full((B,), 64, dtype=torch.int32).cuda()
    q = torch.zeros((B, Hq, 128), dtype=torch.float16).cuda()
    out = torch.zeros((B, Hq, 128), dtype=torch.float32).cuda()
    enc_ws = torch.zeros(max(1, api.nsn_workspace_bytes(shape, api.NSN_OP_ENCODE, B, 64)), dtype=torch.uint8).cuda()
    dec_ws = torch.zeros(max(1, api.nsn_workspace_bytes(shape, api.NSN_OP_DECODE, B)), dtype=torch.uint8).cuda()

    def attend():
        api.nsn_decode_attention_residual(shape, cb, q, kc, vc, coded, L, k_res, v_res, res_len, scale, 0, out=out,
                                          workspace=dec_ws)

    def flush():
        api.nsn_encode(shape, cb, k_res, v_res, coded, full, kc, vc, workspace=enc_ws)

    def set_inputs(i):
        res_len.fill_(1 + 21 * i)
        q.copy_(torch.from_numpy(synth.make_q(62, B, Hq, step=i)))

    eager = []
    for i in range(3):
        set_inputs(i)
        attend()
        torch.cuda.synchronize()
        eager.append(out.clone())
    flush()
    torch.cuda.synchronize()
    flushed = [t.clone() for t in (kc.codes, kc.norms, kc.means, vc.codes, vc.norms, vc.means)]

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        attend()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g_attend, g_flush = torch.cuda.CUDAGraph(), torch.cuda.CUDAGraph()
    with torch.cuda.graph(g_attend):
        attend()
    with torch.cuda.graph(g_flush):
        flush()
    for rep in range(2):
        for i in range(3):
            set_inputs(i)
            g_attend.replay()
            torch.cuda.synchronize()
            assert torch.equal(out, eager[i]), f"replay {rep}/{i} differs from the eager result"
            assert np.isfinite((out * 2).sum().item())   # eager work between replays
        for t in (kc.codes, kc.norms, vc.codes, vc.norms):   # wipe what the flush writes, then replay it
            t[:, :, L * (t.shape[2] // 768):] = 0
        g_flush.replay()
        torch.cuda.synchronize()
        for got, want in zip((kc.codes, kc.norms, kc.means, vc.codes, vc.norms, vc.means), flushed):
            assert torch.equal(got, want), f"flush replay {rep} differs from the eager encode"


def test_full_configuration_step_replays_bit_identically(gpu_api, codebooks):
    """Decode step with everything switched on (un-embedded keys with the mean turned in the kernel, 4-bit
    side information, 64-token groups, residual) and the residual flush, captured and replayed."""
    import torch
    api = gpu_api
    sub, B, Hq, Hkv, L, G = 4, 2, 8, 2, 640, 64
    cb = torch.from_numpy(codebooks[sub].astype(np.float16)).cuda()
    table = api.nsn_build_rope_table(synth.rope_inv_freq(10000.0), 768)
    shape = api.make_shape(sub, Hq, Hkv, 768, G, rope_table=table, side_bits=4)
    kc, vc = api.alloc_cache(shape, B), api.alloc_cache(shape, B)
    k, v = synth.make_kv(63, B, Hkv, L + 64)
    kd, vd = torch.from_numpy(k).cuda(), torch.from_numpy(v).cuda()
    coded = torch.full((B,), L, dtype=torch.int32).cuda()
    api.nsn_encode(shape, cb, kd[:, :, :L].contiguous(), vd[:, :, :L].contiguous(),
                   torch.zeros(B, dtype=torch.int32).cuda(), coded, kc, vc)
    scale = 1.0 / math.sqrt(128)
    k_res, v_res = kd[:, :, L:].contiguous(), vd[:, :, L:].contiguous()
    res_len = torch.zeros(B, dtype=torch.int32).cuda()
    full = torch.full((B,), 64, dtype=torch.int32).cuda()
    q = torch.zeros((B, Hq, 128), dtype=torch.float16).cuda()
    out = torch.zeros((B, Hq, 128), dtype=torch.float32).cuda()
    enc_ws = torch.zeros(max(1, api.nsn_workspace_bytes(shape, api.NSN_OP_ENCODE, B, 64)), dtype=torch.uint8).cuda()
    dec_ws = torch.zeros(max(1, api.nsn_workspace_bytes(shape, api.NSN_OP_DECODE, B)), dtype=torch.uint8).cuda()

    def attend():
        api.nsn_decode_attention_residual(shape, cb, q, kc, vc, coded, L, k_res, v_res, res_len, scale, 0, out=out,
                                          workspace=dec_ws)

    def flush():
        api.nsn_encode(shape, cb, k_res, v_res, coded, full, kc, vc, workspace=enc_ws)

    def set_inputs(i):
        res_len.fill_(1 + 21 * i)
        q.copy_(torch.from_numpy(synth.make_q(63, B, Hq, step=i)))

    eager = []
    for i in range(3):
        set_inputs(i)
        attend()
        torch.cuda.synchronize()
        eager.append(out.clone())
    flush()
    torch.cuda.synchronize()
    flushed = [t.clone() for t in (kc.codes, kc.norms, kc.means, vc.codes, vc.norms, vc.means)]

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        attend()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g_attend, g_flush = torch.cuda.CUDAGraph(), torch.cuda.CUDAGraph()
    with torch.cuda.graph(g_attend):
        attend()
    with torch.cuda.graph(g_flush):
        flush()
    for rep in range(2):
        for i in range(3):
            set_inputs(i)
            g_attend.replay()
            torch.cuda.synchronize()
            assert torch.equal(out, eager[i]), f"replay {rep}/{i} differs from the eager result"
            assert np.isfinite((out * 2).sum().item())   # eager work between replays
        # wipe what the flush writes (block 10 of the sequence: one norms record, one mean record, 64 tokens of codes)
        kc.codes[:, :, L * 32:] = 0
        vc.codes[:, :, L * 32:] = 0
        kc.norms[:, :, L // 64:] = 0
        vc.norms[:, :, L // 64:] = 0
        kc.means[:, :, L // 64:] = 0
        vc.means[:, :, L // 64:] = 0
        g_flush.replay()
        torch.cuda.synchronize()
        for got, want in zip((kc.codes, kc.norms, kc.means, vc.codes, vc.norms, vc.means), flushed):
            assert torch.equal(got, want), f"flush replay {rep} differs from the eager encode"
