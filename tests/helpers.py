"""Test-side helpers: the cache layout written out in numpy from the formulas in include/nsn.h
(independent of the library's own index code), and glue between oracle dictionaries and device
cache buffers."""
from __future__ import annotations

import numpy as np

D = 128


def code_offsets(J: int, kind: str, n_tokens: int, layout: str = "tiled") -> np.ndarray:
    """[n_tokens][J] byte offset inside a placement unit of (token, byte row); the two layouts of include/nsn.h."""
    t, j = np.meshgrid(np.arange(n_tokens), np.arange(J), indexing="ij")
    if layout == "legacy":
        if kind == "k":
            return t * J + j
        return (t // J) * (J * J) + j * J + t % J
    assert layout == "tiled"
    qs, tb = J // 4, t % 64
    if kind == "k":
        lane = 16 * (j // qs) + tb % 16
        return (t // 64) * (64 * J) + lane * J + (tb // 16) * qs + j % qs
    lane = 16 * (tb % 16 // 4) + 4 * (tb % 4) + j % 4
    return (t // 64) * (64 * J) + lane * J + (tb // 16) * qs + j // 4


def pack_codes(codes: np.ndarray, kind: str, capacity: int, layout: str = "tiled") -> np.ndarray:
    """codes u8 [L][J] -> layout bytes u8 [capacity * J] (capacity a multiple of 64 tokens)."""
    L, J = codes.shape
    assert capacity % 64 == 0 and capacity >= L
    full = np.zeros((capacity, J), dtype=np.uint8)
    full[:L] = codes
    out = np.zeros(capacity * J, dtype=np.uint8)
    out[code_offsets(J, kind, capacity, layout).ravel()] = full.ravel()
    return out


def unpack_codes(raw: np.ndarray, kind: str, J: int, layout: str = "tiled") -> np.ndarray:
    """layout bytes u8 [capacity * J] -> codes u8 [capacity][J]."""
    cap = raw.size // J
    return raw[code_offsets(J, kind, cap, layout).ravel()].reshape(cap, J)


def n_groups(length: int, G: int) -> int:
    return (length + G - 1) // G if G > 0 else 1


class HostCache:
    """Numpy mirror of one tensor kind's cache buffers (contiguous or paged)."""

    def __init__(self, kind, batch, hkv, J, max_len, G, page_size=0, block_table=None, n_pages=None,
                 layout="tiled"):
        self.kind, self.batch, self.hkv, self.J, self.max_len, self.G = kind, batch, hkv, J, max_len, G
        self.layout = layout  # "tiled": the (sub_dim, 256) formats without a rope table
        self.page = page_size
        self.bt = block_table
        self.ng = n_groups(max_len, G)
        if page_size:
            pages = n_pages if n_pages is not None else batch * (max_len // page_size)
            self.codes = np.zeros((pages, hkv, page_size * J), dtype=np.uint8)
            self.norms = np.zeros((pages, hkv, page_size, 2), dtype=np.float16)
        else:
            self.codes = np.zeros((batch, hkv, max_len * J), dtype=np.uint8)
            self.norms = np.zeros((batch, hkv, max_len, 2), dtype=np.float16)
        self.means = np.zeros((batch, hkv, self.ng, D), dtype=np.float16)

    def put_unit(self, b, h, enc: dict, start: int = 0, write_means: bool = True):
        """Store an oracle-encoded run of tokens [start, start+L) of unit (b, h)."""
        L = enc["codes"].shape[0]
        if write_means:
            o = enc["o"]
            first = start // self.G if self.G else 0
            if self.G == 0:
                self.means[b, h, 0] = o[0]
            else:
                ng_new = n_groups(L, self.G)
                self.means[b, h, first:first + ng_new] = o[first:first + ng_new]
        logical_codes = self.get_codes(b, h)
        logical_norms = self.get_norms(b, h)
        logical_codes[start:start + L] = enc["codes"]
        logical_norms[start:start + L, 0] = enc["a"]
        logical_norms[start:start + L, 1] = enc["b"]
        self._set_logical(b, h, logical_codes, logical_norms)

    # logical views -------------------------------------------------------------------------
    def get_codes(self, b, h) -> np.ndarray:
        if not self.page:
            return unpack_codes(self.codes[b, h], self.kind, self.J, self.layout)
        parts = [unpack_codes(self.codes[self.bt[b, p], h], self.kind, self.J, self.layout)
                 for p in range(self.max_len // self.page)]
        return np.concatenate(parts, axis=0)

    def get_norms(self, b, h) -> np.ndarray:
        if not self.page:
            return self.norms[b, h].copy()
        return np.concatenate([self.norms[self.bt[b, p], h] for p in range(self.max_len // self.page)], axis=0)

    def _set_logical(self, b, h, codes, norms):
        if not self.page:
            self.codes[b, h] = pack_codes(codes, self.kind, self.max_len, self.layout)
            self.norms[b, h] = norms
            return
        for p in range(self.max_len // self.page):
            sl = slice(p * self.page, (p + 1) * self.page)
            self.codes[self.bt[b, p], h] = pack_codes(codes[sl], self.kind, self.page, self.layout)
            self.norms[self.bt[b, p], h] = norms[sl]

    def unit_dict(self, b, h, length) -> dict:
        """Oracle-style dictionary of the first `length` tokens of unit (b, h)."""
        nm = self.get_norms(b, h)
        return dict(codes=self.get_codes(b, h)[:length], a=nm[:length, 0], b=nm[:length, 1],
                    o=self.means[b, h, :n_groups(length, self.G)])

    # device transfer -----------------------------------------------------------------------
    def to_device(self, api, shape, device="cuda"):
        import torch
        bt = None if self.bt is None else torch.from_numpy(self.bt.astype(np.int32)).to(device)
        return api.CodedCache(torch.from_numpy(self.codes).to(device), torch.from_numpy(self.norms).to(device),
                              torch.from_numpy(self.means).to(device), bt)

    def from_device(self, dc):
        self.codes = dc.codes.cpu().numpy()
        self.norms = dc.norms.cpu().numpy()
        self.means = dc.means.cpu().numpy()


def max_rel_err(out: np.ndarray, ref: np.ndarray) -> float:
    """max_i |out_i - ref_i| / max_i |ref_i| per row, worst row."""
    num = np.abs(out - ref).max(axis=-1)
    den = np.abs(ref).max(axis=-1)
    return float((num / np.maximum(den, 1e-30)).max())


# ---- double quantization (side_bits = 4): the record layouts of include/nsn.h, written out in numpy ----
def _pack_nibbles(codes: np.ndarray) -> np.ndarray:
    """u8 [..., 2n] values 0..15 -> u8 [..., n]; even index = low nibble."""
    return (codes[..., 0::2] | (codes[..., 1::2] << 4)).astype(np.uint8)


def _unpack_nibbles(raw: np.ndarray) -> np.ndarray:
    out = np.empty(raw.shape[:-1] + (raw.shape[-1] * 2,), dtype=np.uint8)
    out[..., 0::2] = raw & 15
    out[..., 1::2] = raw >> 4
    return out


class HostCacheDQ(HostCache):
    """HostCache with 4-bit side information: norms = 164-byte records per 64-token block
    ([0,128) a' fp16, [128,160) s1 codes, [160,164) (min, step) fp16), means = 80-byte records per group
    ([0,64) codes, [64,80) four (min, step) fp16 pairs)."""

    def __init__(self, kind, batch, hkv, J, max_len, G, page_size=0, block_table=None, n_pages=None,
                 layout="tiled"):
        # layout: "tiled" for index-only codes of keys taken as given, "legacy" with sign bytes or a rotary table
        super().__init__(kind, batch, hkv, J, max_len, G, page_size, block_table, n_pages, layout=layout)
        units = self.codes.shape[0]
        per_unit = (page_size or max_len) // 64
        self.norms = np.zeros((units, hkv, per_unit, 164), dtype=np.uint8)
        self.means = np.zeros((batch, hkv, self.ng, 80), dtype=np.uint8)

    # norm records of one (sequence, head) in logical block order: [max_len / 64][164]
    def _records(self, b, h) -> np.ndarray:
        if not self.page:
            return self.norms[b, h].copy()
        return np.concatenate([self.norms[self.bt[b, p], h] for p in range(self.max_len // self.page)], axis=0)

    def _set_records(self, b, h, rec):
        if not self.page:
            self.norms[b, h] = rec
            return
        per = self.page // 64
        for p in range(self.max_len // self.page):
            self.norms[self.bt[b, p], h] = rec[p * per:(p + 1) * per]

    def put_unit(self, b, h, enc: dict, start: int = 0, write_means: bool = True):
        L = enc["codes"].shape[0]
        assert start % 64 == 0
        if write_means:
            first = start // self.G if self.G else 0
            ng_new = n_groups(L, self.G) if self.G else 1
            for gi in range(first, first + ng_new):
                self.means[b, h, gi, :64] = _pack_nibbles(enc["o_code"][gi])
                self.means[b, h, gi, 64:] = enc["o_par"][gi].astype(np.float16).reshape(-1).view(np.uint8)
        logical_codes = self.get_codes(b, h)
        logical_codes[start:start + L] = enc["codes"]
        rec = self._records(b, h)
        a_all = rec[:, :128].copy().view(np.float16).reshape(-1)
        c_all = _unpack_nibbles(rec[:, 128:160]).reshape(-1)
        a_all[start:start + L] = enc["a_stored"]
        c_all[start:start + L] = enc["b_code"]
        rec[:, :128] = a_all.reshape(-1, 64).view(np.uint8)
        rec[:, 128:160] = _pack_nibbles(c_all.reshape(-1, 64))
        for blk in range(start // 64, (start + L + 63) // 64):
            rec[blk, 160:164] = enc["b_par"][blk].astype(np.float16).view(np.uint8)
        self._set_records(b, h, rec)
        if not self.page:
            self.codes[b, h] = pack_codes(logical_codes, self.kind, self.max_len, self.layout)
        else:
            for p in range(self.max_len // self.page):
                self.codes[self.bt[b, p], h] = pack_codes(logical_codes[p * self.page:(p + 1) * self.page], self.kind,
                                                          self.page, self.layout)

    def unit_dict(self, b, h, length) -> dict:
        """Effective float64 a, b, o (what the decoder reconstructs) plus the stored fields."""
        rec = self._records(b, h)
        a_stored = rec[:, :128].copy().view(np.float16).reshape(-1)[:length]
        b_code = _unpack_nibbles(rec[:, 128:160]).reshape(-1)[:length]
        b_par = rec[:, 160:164].copy().view(np.float16).reshape(-1, 2)
        blk = np.arange(length) // 64
        b_hat = b_par[blk, 0].astype(np.float64) + b_par[blk, 1].astype(np.float64) * b_code
        ng = n_groups(length, self.G)
        o_code = _unpack_nibbles(self.means[b, h, :ng, :64])
        o_par = self.means[b, h, :ng, 64:].copy().view(np.float16).reshape(ng, 4, 2)
        o_hat = (np.repeat(o_par[:, :, 0].astype(np.float64), 32, axis=1) +
                 np.repeat(o_par[:, :, 1].astype(np.float64), 32, axis=1) * o_code)
        return dict(codes=self.get_codes(b, h)[:length], a=b_hat * a_stored.astype(np.float64), b=b_hat, o=o_hat,
                    a_stored=a_stored, b_code=b_code, b_par=b_par[:(length + 63) // 64], o_code=o_code, o_par=o_par)
