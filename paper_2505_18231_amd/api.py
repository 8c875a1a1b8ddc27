"""Thin ctypes binding of libnsn.so (same names as include/nsn.h).

Argument marshalling only: every step of the path runs inside the HIP kernels.  PyTorch is
used for device memory and the current stream.  There is no CPU fallback: a missing library
raises at import of the first call.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libnsn.so")

NSN_OK = 0
NSN_ERR_INVALID_ARG, NSN_ERR_UNSUPPORTED, NSN_ERR_WORKSPACE, NSN_ERR_HIP = -1, -2, -3, -4
NSN_OP_ENCODE, NSN_OP_DECODE, NSN_OP_CODEBOOK = 0, 1, 2
NSN_VARIANT_DEFAULT, NSN_VARIANT_ALT = 0, 1
HEAD_DIM, N_CODES = 128, 256


class nsn_shape(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("head_dim", "sub_dim", "n_codes", "n_q_heads", "n_kv_heads",
                                         "group_size", "page_size", "max_len")] + [("rope_table", C.c_void_p),
                                                                                     ("side_bits", C.c_int32)]


class nsn_cache(C.Structure):
    _fields_ = [("codes", C.c_void_p), ("norms", C.c_void_p), ("means", C.c_void_p),
                ("block_table", C.c_void_p)]


class nsn_residual(C.Structure):
    _fields_ = [("k_fp16", C.c_void_p), ("v_fp16", C.c_void_p), ("lens", C.c_void_p), ("capacity", C.c_int32)]


class NsnError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"libnsn error {code}: {text}")
        self.code = code


_lib = None


def lib() -> C.CDLL:
    """Load libnsn.so (built in-tree by paper_2505_18231_amd.build); fail loudly if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2505_18231_amd.build` "
                "(there is no CPU fallback)")
        L = C.CDLL(LIB_PATH)
        L.nsn_last_error.restype = C.c_char_p
        L.nsn_workspace_bytes.restype = C.c_size_t
        L.nsn_workspace_bytes.argtypes = [C.POINTER(nsn_shape), C.c_int, C.c_int, C.c_int64, C.c_int]
        L.nsn_max_groups.argtypes = [C.POINTER(nsn_shape)]
        L.nsn_select_variant.argtypes = [C.c_int, C.c_int]
        for fn in (L.nsn_k_code_offset, L.nsn_v_code_offset):
            fn.restype = C.c_int64
            fn.argtypes = [C.POINTER(nsn_shape), C.c_int64, C.c_int]
        L.nsn_build_codebook.argtypes = [C.c_void_p, C.c_int64, C.c_int, C.c_int, C.c_int, C.c_void_p,
                                         C.POINTER(C.c_double), C.c_void_p, C.c_size_t, C.c_void_p]
        L.nsn_finetune_codebook.argtypes = [C.c_void_p, C.c_int64, C.c_int, C.c_int, C.c_int, C.c_double,
                                            C.c_void_p, C.POINTER(C.c_double), C.c_void_p, C.c_size_t, C.c_void_p]
        L.nsn_quantize_codebook.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p]
        L.nsn_rope_table_bytes.restype = C.c_size_t
        L.nsn_rope_table_bytes.argtypes = [C.c_int]
        L.nsn_build_rope_table.argtypes = [C.POINTER(C.c_float), C.c_int, C.c_void_p, C.c_size_t, C.c_void_p]
        L.nsn_encode.argtypes = [C.POINTER(nsn_shape), C.c_void_p, C.c_void_p, C.c_void_p, C.c_int,
                                 C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.POINTER(nsn_cache),
                                 C.POINTER(nsn_cache), C.c_void_p, C.c_size_t, C.c_void_p]
        L.nsn_decode_attention.argtypes = [C.POINTER(nsn_shape), C.c_void_p, C.c_void_p,
                                           C.POINTER(nsn_cache), C.POINTER(nsn_cache), C.c_void_p, C.c_int,
                                           C.c_int, C.c_float, C.c_int, C.c_void_p, C.c_void_p, C.c_size_t,
                                           C.c_void_p]
        L.nsn_decode_attention_residual.argtypes = [
            C.POINTER(nsn_shape), C.c_void_p, C.c_void_p, C.POINTER(nsn_cache), C.POINTER(nsn_cache), C.c_void_p,
            C.c_int, C.c_int, C.POINTER(nsn_residual), C.c_float, C.c_int, C.c_void_p, C.c_void_p, C.c_size_t,
            C.c_void_p]
        L.nsn_decode_attention_noalloc.argtypes = [C.POINTER(nsn_shape), C.c_void_p, C.c_void_p,
                                                   C.POINTER(nsn_cache), C.POINTER(nsn_cache), C.c_void_p, C.c_int,
                                                   C.c_int, C.c_float, C.c_int, C.c_void_p, C.c_void_p]
        _lib = L
    return _lib


def _check(rc: int) -> None:
    if rc != NSN_OK:
        raise NsnError(rc, lib().nsn_last_error().decode())


def _ptr(t) -> int | None:
    return None if t is None else t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


SIGN_CODES = 65536  # n_codes of the sign + index format: 256 magnitude codewords x 2^8 sign patterns


def make_shape(sub_dim: int, n_q_heads: int, n_kv_heads: int, max_len: int, group_size: int = 0,
               page_size: int = 0, sign_format: bool = False, rope_table: torch.Tensor | None = None,
               side_bits: int = 16) -> nsn_shape:
    """sign_format: the paper's 2-bit format (8 sign bits + 8-bit index per 8-dim sub-vector).
    rope_table: result of nsn_build_rope_table - keys are normalised before the rotary embedding.
    side_bits: 4 = double quantization of the first-Normalize scales and the group means."""
    assert not sign_format or sub_dim == 8
    shape = nsn_shape(HEAD_DIM, sub_dim, SIGN_CODES if sign_format else N_CODES, n_q_heads, n_kv_heads, group_size,
                      page_size, max_len, _ptr(rope_table), side_bits)
    shape._rope_keepalive = rope_table  # the struct only holds the address
    return shape


def nsn_build_rope_table(inv_freq, max_len: int, device="cuda") -> torch.Tensor:
    """inv_freq: 64 fp32 values (host).  Returns the device table (uint8) for positions < max_len."""
    import numpy as np
    f = np.ascontiguousarray(np.asarray(inv_freq, dtype=np.float32))
    assert f.shape == (HEAD_DIM // 2,)
    need = lib().nsn_rope_table_bytes(max_len)
    assert need > 0, "max_len must be a positive multiple of 64"
    table = torch.empty(need, dtype=torch.uint8, device=device)
    _check(lib().nsn_build_rope_table(f.ctypes.data_as(C.POINTER(C.c_float)), max_len, table.data_ptr(), need,
                                      _stream()))
    return table


def code_bytes_per_token(shape: nsn_shape) -> int:
    return (2 if shape.n_codes == SIGN_CODES else 1) * (HEAD_DIM // shape.sub_dim)


def nsn_max_groups(shape: nsn_shape) -> int:
    return lib().nsn_max_groups(C.byref(shape))


def nsn_select_variant(op: int, variant: int) -> int:
    """Process-wide kernel variant of NSN_OP_ENCODE / NSN_OP_DECODE; returns the previous one."""
    prev = lib().nsn_select_variant(op, variant)
    _check(min(prev, 0))
    return prev


def nsn_workspace_bytes(shape: nsn_shape, op: int, batch: int, n: int = 0, n_splits: int = 0) -> int:
    return lib().nsn_workspace_bytes(C.byref(shape), op, batch, n, n_splits)


@dataclass
class CodedCache:
    """Device buffers of one tensor kind (K or V) in the layout include/nsn.h documents."""
    codes: torch.Tensor          # uint8
    norms: torch.Tensor          # fp16 [..., 2] = (a, b)
    means: torch.Tensor          # fp16 [B][Hkv][NG][128]
    block_table: torch.Tensor | None

    def c_struct(self) -> nsn_cache:
        return nsn_cache(self.codes.data_ptr(), self.norms.data_ptr(), self.means.data_ptr(),
                         _ptr(self.block_table))


def alloc_cache(shape: nsn_shape, batch: int, device="cuda", block_table: torch.Tensor | None = None,
                n_pages: int | None = None) -> CodedCache:
    """Zero-initialised cache buffers.  Paged layout: n_pages physical pages (default: enough for all)."""
    J = code_bytes_per_token(shape)
    hkv = shape.n_kv_heads
    ng = nsn_max_groups(shape)
    dq = shape.side_bits == 4   # norms: 164-byte records per 64 tokens; means: 80-byte records
    if shape.page_size > 0:
        pages = n_pages if n_pages is not None else batch * (shape.max_len // shape.page_size)
        codes = torch.zeros((pages, hkv, shape.page_size * J), dtype=torch.uint8, device=device)
        norms = (torch.zeros((pages, hkv, shape.page_size // 64, 164), dtype=torch.uint8, device=device) if dq else
                 torch.zeros((pages, hkv, shape.page_size, 2), dtype=torch.float16, device=device))
        assert block_table is not None and block_table.dtype == torch.int32
    else:
        codes = torch.zeros((batch, hkv, shape.max_len * J), dtype=torch.uint8, device=device)
        norms = (torch.zeros((batch, hkv, shape.max_len // 64, 164), dtype=torch.uint8, device=device) if dq else
                 torch.zeros((batch, hkv, shape.max_len, 2), dtype=torch.float16, device=device))
    means = (torch.zeros((batch, hkv, ng, 80), dtype=torch.uint8, device=device) if dq else
             torch.zeros((batch, hkv, ng, HEAD_DIM), dtype=torch.float16, device=device))
    return CodedCache(codes, norms, means, block_table)


def nsn_build_codebook(samples: torch.Tensor, n_codes: int = N_CODES, iters: int = 50,
                       workspace: torch.Tensor | None = None):
    """samples: cuda fp32 [n][sub_dim].  Returns (codebook cuda fp16 [n_codes][sub_dim], mse per dim)."""
    assert samples.is_cuda and samples.dtype == torch.float32 and samples.is_contiguous()
    n, sub = samples.shape
    shp = make_shape(sub, 1, 1, 64)
    need = nsn_workspace_bytes(shp, NSN_OP_CODEBOOK, 1, n)
    if workspace is None:
        workspace = torch.empty(max(need, 1), dtype=torch.uint8, device=samples.device)
    codebook = torch.empty((n_codes, sub), dtype=torch.float16, device=samples.device)
    mse = C.c_double(0.0)
    _check(lib().nsn_build_codebook(samples.data_ptr(), n, sub, n_codes, iters, codebook.data_ptr(),
                                    C.byref(mse), workspace.data_ptr(), workspace.numel(), _stream()))
    return codebook, mse.value


def nsn_finetune_codebook(samples: torch.Tensor, codebook: torch.Tensor, iters: int, lr: float,
                          workspace: torch.Tensor | None = None):
    """samples: cuda fp32 [n][sub_dim]; codebook: cuda fp16 [256][sub_dim], updated in place.
    Returns (codebook, mean cosine similarity before, after)."""
    assert samples.is_cuda and samples.dtype == torch.float32 and samples.is_contiguous()
    assert codebook.is_cuda and codebook.dtype == torch.float16 and codebook.is_contiguous()
    n, sub = samples.shape
    assert codebook.shape == (N_CODES, sub)
    need = nsn_workspace_bytes(make_shape(sub, 1, 1, 64), NSN_OP_CODEBOOK, 1, n)
    if workspace is None:
        workspace = torch.empty(max(need, 1), dtype=torch.uint8, device=samples.device)
    cos = (C.c_double * 2)(0.0, 0.0)
    _check(lib().nsn_finetune_codebook(samples.data_ptr(), n, sub, N_CODES, iters, float(lr), codebook.data_ptr(),
                                       cos, workspace.data_ptr(), workspace.numel(), _stream()))
    return codebook, cos[0], cos[1]


def nsn_quantize_codebook(codebook: torch.Tensor):
    """codebook: cuda fp16 [256][sub_dim], snapped in place to 16 levels.
    Returns (codebook, codes cuda u8 [256][sub_dim], levels cuda fp16 [2] = (min, step))."""
    assert codebook.is_cuda and codebook.dtype == torch.float16 and codebook.is_contiguous()
    n, sub = codebook.shape
    codes = torch.empty((n, sub), dtype=torch.uint8, device=codebook.device)
    levels = torch.empty(2, dtype=torch.float16, device=codebook.device)
    _check(lib().nsn_quantize_codebook(codebook.data_ptr(), sub, n, codes.data_ptr(), levels.data_ptr(), _stream()))
    return codebook, codes, levels


def nsn_encode(shape: nsn_shape, codebook: torch.Tensor, k: torch.Tensor, v: torch.Tensor,
               seq_start: torch.Tensor, n_new: torch.Tensor, k_cache: CodedCache, v_cache: CodedCache,
               freeze_means: bool = False, workspace: torch.Tensor | None = None) -> None:
    """k, v: cuda fp16 [B][Hkv][max_new][128]; seq_start, n_new: cuda int32 [B]."""
    assert k.is_cuda and k.dtype == torch.float16 and k.is_contiguous() and k.shape == v.shape
    assert v.dtype == torch.float16 and v.is_contiguous()
    assert codebook.dtype == torch.float16 and codebook.is_contiguous()
    assert seq_start.dtype == torch.int32 and n_new.dtype == torch.int32
    batch, hkv, max_new, d = k.shape
    assert hkv == shape.n_kv_heads and d == HEAD_DIM
    need = nsn_workspace_bytes(shape, NSN_OP_ENCODE, batch, max_new)
    if workspace is None:
        workspace = torch.empty(max(need, 1), dtype=torch.uint8, device=k.device)
    kc, vc = k_cache.c_struct(), v_cache.c_struct()
    _check(lib().nsn_encode(C.byref(shape), codebook.data_ptr(), k.data_ptr(), v.data_ptr(), max_new,
                            seq_start.data_ptr(), n_new.data_ptr(), batch, int(freeze_means),
                            C.byref(kc), C.byref(vc), workspace.data_ptr(), workspace.numel(), _stream()))


def nsn_decode_attention(shape: nsn_shape, codebook: torch.Tensor, q: torch.Tensor, k_cache: CodedCache,
                         v_cache: CodedCache, seq_lens: torch.Tensor, max_seq_len: int,
                         softmax_scale: float, n_splits: int = 0, out: torch.Tensor | None = None,
                         workspace: torch.Tensor | None = None) -> torch.Tensor:
    """q: cuda fp16 [B][Hq][128]; returns cuda fp32 [B][Hq][128]."""
    assert q.is_cuda and q.dtype == torch.float16 and q.is_contiguous()
    assert seq_lens.dtype == torch.int32 and codebook.dtype == torch.float16
    batch, hq, d = q.shape
    assert hq == shape.n_q_heads and d == HEAD_DIM
    if out is None:
        out = torch.empty((batch, hq, d), dtype=torch.float32, device=q.device)
    need = nsn_workspace_bytes(shape, NSN_OP_DECODE, batch, 0, n_splits)
    if workspace is None:  # must start zero-filled (arrival counters); reusable afterwards
        workspace = torch.zeros(max(need, 1), dtype=torch.uint8, device=q.device)
    kc, vc = k_cache.c_struct(), v_cache.c_struct()
    _check(lib().nsn_decode_attention(C.byref(shape), codebook.data_ptr(), q.data_ptr(), C.byref(kc),
                                      C.byref(vc), seq_lens.data_ptr(), batch, max_seq_len,
                                      float(softmax_scale), n_splits, out.data_ptr(), workspace.data_ptr(),
                                      workspace.numel(), _stream()))
    return out


def nsn_decode_attention_residual(shape: nsn_shape, codebook: torch.Tensor, q: torch.Tensor,
                                  k_cache: CodedCache, v_cache: CodedCache, seq_lens: torch.Tensor,
                                  max_seq_len: int, k_res: torch.Tensor, v_res: torch.Tensor,
                                  res_lens: torch.Tensor, softmax_scale: float, n_splits: int = 0,
                                  out: torch.Tensor | None = None,
                                  workspace: torch.Tensor | None = None) -> torch.Tensor:
    """As nsn_decode_attention, plus the fp16 residual k_res, v_res: cuda fp16 [B][Hkv][capacity][128]
    with res_lens (cuda int32 [B]) valid rows each; seq_lens counts the coded tokens only."""
    assert q.is_cuda and q.dtype == torch.float16 and q.is_contiguous()
    assert seq_lens.dtype == torch.int32 and res_lens.dtype == torch.int32 and codebook.dtype == torch.float16
    batch, hq, d = q.shape
    assert hq == shape.n_q_heads and d == HEAD_DIM
    for t in (k_res, v_res):
        assert t.is_cuda and t.dtype == torch.float16 and t.is_contiguous()
        assert t.dim() == 4 and t.shape[0] == batch and t.shape[1] == shape.n_kv_heads and t.shape[3] == HEAD_DIM
    assert k_res.shape == v_res.shape and res_lens.numel() == batch
    if out is None:
        out = torch.empty((batch, hq, d), dtype=torch.float32, device=q.device)
    need = nsn_workspace_bytes(shape, NSN_OP_DECODE, batch, 0, n_splits)
    if workspace is None:
        workspace = torch.zeros(max(need, 1), dtype=torch.uint8, device=q.device)
    kc, vc = k_cache.c_struct(), v_cache.c_struct()
    res = nsn_residual(k_res.data_ptr(), v_res.data_ptr(), res_lens.data_ptr(), int(k_res.shape[2]))
    _check(lib().nsn_decode_attention_residual(C.byref(shape), codebook.data_ptr(), q.data_ptr(), C.byref(kc),
                                               C.byref(vc), seq_lens.data_ptr(), batch, max_seq_len,
                                               C.byref(res), float(softmax_scale), n_splits, out.data_ptr(),
                                               workspace.data_ptr(), workspace.numel(), _stream()))
    return out


def nsn_decode_attention_noalloc(shape: nsn_shape, codebook: torch.Tensor, q: torch.Tensor, k_cache: CodedCache,
                                 v_cache: CodedCache, seq_lens: torch.Tensor, max_seq_len: int,
                                 softmax_scale: float, n_splits: int = 0, out: torch.Tensor | None = None) -> torch.Tensor:
    """nsn_decode_attention without a workspace: scratch is a fixed array inside the library (4 MiB per GPU)."""
    assert q.is_cuda and q.dtype == torch.float16 and q.is_contiguous()
    assert seq_lens.dtype == torch.int32 and codebook.dtype == torch.float16
    batch, hq, d = q.shape
    assert hq == shape.n_q_heads and d == HEAD_DIM and out is not None, "pass `out`: this entry point allocates nothing"
    kc, vc = k_cache.c_struct(), v_cache.c_struct()
    _check(lib().nsn_decode_attention_noalloc(C.byref(shape), codebook.data_ptr(), q.data_ptr(), C.byref(kc),
                                              C.byref(vc), seq_lens.data_ptr(), batch, max_seq_len,
                                              float(softmax_scale), n_splits, out.data_ptr(), _stream()))
    return out
