"""CPU oracle for the NSNQuant coded-KV hot path (arXiv 2505.18231).

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition the HIP path is
checked against.  Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline
leg may import it; the product package never does, and nothing here imports the
product package.  Everything is numpy float64 unless a storage rounding point is
named.  No blocking, fusion, lookup tables (except `lut_scores`, which exists to
prove the table form equals the definition) or online softmax.

Parity pins (tests/test_oracle_*.py, all CPU):
  hadamard            H H^T = I, H = H^T, |entries| = 1/sqrt(d), Sylvester doubling
  nsn                 token norms sqrt(d) after both Normalize steps, zero channel
                      mean after Shift, restore identity v = s1 (s2 v_nsn + o),
                      NSN and the rotation commute (Sec. 3.2)
  nearest_codeword    the paper's 2-d worked example (App. C.3), exhaustive search
                      written as an independent python loop on tiny inputs
  scale adjustment    worked example factor 1.25; (alpha v_Q - v) . v = 0 (Sec. 3.3)
  encode / dequantize round trip error orthogonal to the rotated token; bit budget
                      2.5 bits of Table 11's baseline row
  decode_attention    equals lut_scores + softmax form; L = 1 gives the dequantised
                      value token; equal scores give the mean value token
  build_codebook      Lloyd inertia never increases; final per-dimension distortion
                      lies between the Gaussian rate-distortion bound and the
                      product scalar Lloyd-Max quantiser.  The centroid values
                      themselves are "parity unpinned" against the paper (its tuned
                      codebook is not printed); GPU and oracle are compared with
                      one and the same codebook array.
  decode_attention_residual   no residual = coded-only attention; no coded tokens = plain
                      softmax attention written with loops; both = merge of the two by
                      their softmax masses (Sec. 3.2 "Residual")
  sign + index format the (signs, nearest magnitude codeword) pair equals the exhaustive Eq. 1
                      search over all 256 x 2^8 signed codewords on small inputs; 16 bits per
                      8 dims; round trip keeps the scale-adjustment orthogonality.  How the
                      paper builds its magnitude codebook is not described: K-Means on |N(0,1)|
                      samples is this build's reading ("parity unpinned" for the codebook)
  finetune_codebook   gradient equals central finite differences of the cosine loss at a
                      fixed assignment and is orthogonal to its codeword; the cosine
                      similarity rises.  Optimiser, rate and step count are this build's
                      reading: "parity unpinned" against the paper's tuned codebook (Sec. 3.4)
  rope / pre-RoPE keys   a hand-computed 4-channel rotation (fixes pairing and sense of rotation);
                      complex-multiplication form; scores depend on the position difference only;
                      zero frequencies reduce encode / decode to the plain path; the restore
                      identity RoPE(x) = s1 (s2 RoPE(v_nsn) + RoPE(o)); App. B's two-branch score
                      with the query turned back instead of the mean turned forward.  Pairing,
                      frequencies and positions are this build's reading (the paper names its
                      models' RoPE without restating it)
  double quantization rtn4 reproduces an exactly representable 16-level grid, its error is at most
                      half a step, a constant group gives step 0; the bit budget reproduces
                      Table 11's 2.33 and 2.23 (printed to two decimals); with 4-bit side
                      information encode / dequantize keep the restore identity with the
                      dequantised scale and mean.  Min/max (asymmetric) levels with fp16 minimum and
                      step are this build's reading of "4-bit round-to-nearest"
"""
from __future__ import annotations

import numpy as np

F64 = np.float64


# ----------------------------------------------------------------------------
# storage rounding
# ----------------------------------------------------------------------------
def fp16_rne(x) -> np.ndarray:
    """Round float64 to the nearest fp16 (ties to even) in ONE rounding, return as fp16."""
    return np.asarray(x, dtype=F64).astype(np.float16)


# ----------------------------------------------------------------------------
# Hadamard transform (Sec. 2 "Hadamard transform"; App. A.1 step 3: rows h = s / sqrt(d))
# ----------------------------------------------------------------------------
def hadamard(d: int) -> np.ndarray:
    """Orthonormal Sylvester Hadamard matrix, natural order, no random signs."""
    assert d >= 1 and (d & (d - 1)) == 0
    h = np.ones((1, 1), dtype=F64)
    while h.shape[0] < d:
        h = np.block([[h, h], [h, -h]])
    return h / np.sqrt(F64(d))


# ----------------------------------------------------------------------------
# Normalize - Shift - Normalize, exactly as the three numbered steps of Sec. 3.2
# (no storage rounding; used by the pins and by `encode` below)
# ----------------------------------------------------------------------------
def _safe_div(num: np.ndarray, den: np.ndarray) -> np.ndarray:
    """num / den with the reading 'a zero scale gives a zero vector'."""
    den = np.asarray(den, dtype=F64)
    out = np.zeros_like(num, dtype=F64)
    np.divide(num, den, out=out, where=(den != 0))
    return out


def token_scale(v: np.ndarray) -> np.ndarray:
    """norm(v, per token) / sqrt(d)  (steps 1 and 3 of Sec. 3.2)."""
    d = v.shape[-1]
    return np.sqrt(np.sum(v * v, axis=-1)) / np.sqrt(F64(d))


def group_index(n_tokens: int, group_size: int, start: int = 0) -> np.ndarray:
    """Shift group of each token: absolute position // G, or 0 when G == 0 (one group)."""
    t = np.arange(start, start + n_tokens)
    return (t // group_size) if group_size > 0 else np.zeros(n_tokens, dtype=np.int64)


def nsn(v: np.ndarray, group_size: int = 0):
    """Sec. 3.2 steps 1-3 on v [l][d]; returns (s1 [l], o [n_groups][d], s2 [l], v_nsn [l][d]).

    The Shift mean is taken per channel over the tokens of one group (the residual-size
    chunks of Sec. 3.2 'Residual'); group_size 0 means a single group.
    """
    v = np.asarray(v, dtype=F64)
    s1 = token_scale(v)
    vn = _safe_div(v, s1[:, None])
    g = group_index(v.shape[0], group_size)
    ng = int(g.max()) + 1 if v.shape[0] else 0
    o = np.zeros((ng, v.shape[1]), dtype=F64)
    for gi in range(ng):
        o[gi] = vn[g == gi].mean(axis=0)
    vns = vn - o[g]
    s2 = token_scale(vns)
    vnsn = _safe_div(vns, s2[:, None])
    return s1, o, s2, vnsn


def nsn_restore(s1, o, s2, vnsn, group_size: int = 0):
    """v = s1 (s2 v_nsn + o)  (Sec. 3.2, sentence after the enumerated steps)."""
    g = group_index(vnsn.shape[0], group_size)
    return s1[:, None] * (s2[:, None] * vnsn + o[g])


# ----------------------------------------------------------------------------
# Vector quantisation, Eq. (1): VQ(v) = argmin_i D(v, C[i]),  D = squared Euclidean
# ----------------------------------------------------------------------------
def nearest_codeword(x: np.ndarray, codebook: np.ndarray, chunk: int = 32768):
    """For each row of x [n][sub]: index of the nearest codeword (lowest index on ties),
    plus the best and second-best squared distances (for the tests' tie window)."""
    x = np.asarray(x, dtype=F64)
    c = np.asarray(codebook, dtype=F64)
    n, sub = x.shape
    idx = np.empty(n, dtype=np.int64)
    best = np.empty(n, dtype=F64)
    second = np.empty(n, dtype=F64)
    for s in range(0, n, chunk):
        xs = x[s:s + chunk]
        dist = np.zeros((xs.shape[0], c.shape[0]), dtype=F64)
        for i in range(sub):
            diff = xs[:, i:i + 1] - c[None, :, i]
            dist += diff * diff
        k = np.argmin(dist, axis=1)  # first occurrence = lowest index on ties
        idx[s:s + chunk] = k
        rows = np.arange(xs.shape[0])
        best[s:s + chunk] = dist[rows, k]
        if c.shape[0] > 1:
            dist[rows, k] = np.inf
            second[s:s + chunk] = dist.min(axis=1)
        else:
            second[s:s + chunk] = np.inf
    return idx, best, second


def scale_adjust(v: np.ndarray, vq: np.ndarray) -> np.ndarray:
    """Sec. 3.3: factor ||v||^2 / (v . v_Q) per row; 1 where v . v_Q is not positive."""
    d = v.shape[-1]
    dot = np.sum(v * vq, axis=-1)
    nrm2 = np.sum(v * v, axis=-1)
    alpha = np.ones_like(dot)
    ok = dot > 1e-12 * d
    alpha[ok] = nrm2[ok] / dot[ok]
    return alpha


# ----------------------------------------------------------------------------
# Double quantization (Sec. 3.5): the side information itself is stored in 4 bits, round-to-nearest
# on 16 levels between a group's minimum and maximum; the minimum and the step are kept in fp16.
# Groups: 32 channels of a mean vector o; the s1 of the 64 tokens of one residual-size chunk.
# ----------------------------------------------------------------------------
def rtn4_encode(x):
    """One group of values -> (codes u8 in 0..15, minimum fp16, step fp16).  The codes are taken
    against the ROUNDED minimum and step (what the decoder will see); a zero step gives code 0."""
    x = np.asarray(x, dtype=F64).reshape(-1)
    mn = fp16_rne(x.min())
    st = fp16_rne((x.max() - x.min()) / 15.0)
    if float(st) == 0.0:
        return np.zeros(x.shape, dtype=np.uint8), mn, st
    lvl = np.floor((x - float(mn)) / float(st) + 0.5)
    return np.clip(lvl, 0, 15).astype(np.uint8), mn, st


def rtn4_decode(codes, mn, st) -> np.ndarray:
    return float(mn) + float(st) * np.asarray(codes, dtype=F64)


def quantize_codebook_4bit(codebook):
    """Sec. 3.5, last sentence: the codebook entries themselves on 16 levels.  The grouping is not
    stated; one (minimum, step) pair for the whole codebook is this build's reading.  Returns the
    codebook as the kernels see it (every entry = fp16(min + step * code)) and the codes."""
    c = np.asarray(codebook, dtype=F64)
    code, mn, st = rtn4_encode(c.reshape(-1))
    vals = fp16_rne(rtn4_decode(code, mn, st)).astype(F64).reshape(c.shape)
    return vals, code.reshape(c.shape), mn, st


def quantize_side_info(b16: np.ndarray, o_mean: np.ndarray, start: int = 0):
    """b16 fp16 [l] (first-Normalize scales of tokens start.., start a multiple of 64),
    o_mean float64 [n_groups][d] (rows that are all zero are groups without tokens).
    Returns dict(b_code u8 [l], b_par fp16 [n_blocks][2] (min, step) indexed by absolute 64-token block,
                 o_code u8 [n_groups][d], o_par fp16 [n_groups][d/32][2],
                 b_hat float64 [l], o_hat float64 [n_groups][d])."""
    assert start % 64 == 0
    l = b16.shape[0]
    n_blk = (start + l + 63) // 64
    b_code = np.zeros(l, dtype=np.uint8)
    b_par = np.zeros((n_blk, 2), dtype=np.float16)
    b_hat = np.zeros(l, dtype=F64)
    for blk in range(start // 64, n_blk):
        lo, hi = blk * 64 - start, min((blk + 1) * 64 - start, l)
        code, mn, st = rtn4_encode(b16[lo:hi].astype(F64))
        b_code[lo:hi], b_par[blk] = code, (mn, st)
        b_hat[lo:hi] = rtn4_decode(code, mn, st)
    ng, d = o_mean.shape
    o_code = np.zeros((ng, d), dtype=np.uint8)
    o_par = np.zeros((ng, d // 32, 2), dtype=np.float16)
    o_hat = np.zeros((ng, d), dtype=F64)
    for gi in range(ng):
        for c in range(d // 32):
            sl = slice(32 * c, 32 * c + 32)
            code, mn, st = rtn4_encode(o_mean[gi, sl])
            o_code[gi, sl], o_par[gi, c] = code, (mn, st)
            o_hat[gi, sl] = rtn4_decode(code, mn, st)
    return dict(b_code=b_code, b_par=b_par, o_code=o_code, o_par=o_par, b_hat=b_hat, o_hat=o_hat)


# ----------------------------------------------------------------------------
# Rotary position embedding as the Llama-family models of the paper's experiments apply it:
# channel i and channel i + d/2 form a pair that turns by the angle position * inv_freq[i].
# Sec. 3.2 ("NSN applied to key and value") normalises keys BEFORE this rotation: the rotation
# is applied to v_nsn on the way into the quantiser and to the stored mean o inside the score
# computation (App. B).
# ----------------------------------------------------------------------------
def rope(x: np.ndarray, positions, inv_freq) -> np.ndarray:
    """Rows of x [l][d] rotated by their positions [l]; inv_freq [d/2] (radians per position)."""
    x = np.asarray(x, dtype=F64)
    half = x.shape[1] // 2
    ang = np.asarray(positions, dtype=F64)[:, None] * np.asarray(inv_freq, dtype=F64)[None, :]
    c, s = np.cos(ang), np.sin(ang)
    out = np.empty_like(x)
    out[:, :half] = x[:, :half] * c - x[:, half:] * s
    out[:, half:] = x[:, half:] * c + x[:, :half] * s
    return out


# ----------------------------------------------------------------------------
# Encoder: NSN -> Hadamard -> VQ -> scale adjustment, with the three fp16 storage
# rounding points (b = s1, o, a = s1 s2 alpha); rounded b and o are the values used
# downstream, so that dequantisation is self-consistent.
# ----------------------------------------------------------------------------
def shift_stats(x16: np.ndarray, group_size: int = 0, start: int = 0, given_b=None, given_o=None,
                raw_mean: bool = False):
    """Stage A of the encoder: b = fp16(s1) per token (step 1 of Sec. 3.2) and o = fp16(per-group
    channel mean of x / b) (step 2).  `given_*` replace the computed arrays.  raw_mean: return the
    float64 means before any storage rounding (the input of the 4-bit quantiser of Sec. 3.5)."""
    x = np.asarray(x16, dtype=F64)
    l, d = x.shape
    b16 = fp16_rne(token_scale(x)) if given_b is None else np.asarray(given_b, dtype=np.float16)
    if given_o is not None:
        return b16, np.asarray(given_o, dtype=np.float16)
    assert group_size == 0 or start % group_size == 0, "a new group starts on a boundary"
    assert group_size != 0 or start == 0
    n = _safe_div(x, b16.astype(F64)[:, None])
    g = group_index(l, group_size, start)
    o16 = np.zeros(((int(g.max()) + 1) if l else 0, d), dtype=F64 if raw_mean else np.float16)
    for gi in np.unique(g):
        m = n[g == gi].mean(axis=0)
        o16[gi] = m if raw_mean else fp16_rne(m)
    return b16, o16


# The paper's own 2-bit format (Sec. 3.4): an 8-dim sub-vector is stored as 8 sign bits plus the
# 8-bit index of a codeword with non-negative entries (a codebook of magnitudes); the implied
# codebook holds the 256 x 2^8 signed versions, and because the magnitudes are non-negative the
# nearest of those (Eq. 1) takes the signs of the sub-vector itself and the magnitude codeword
# nearest to its absolute values.  Bit i of the sign byte is set when entry i is negative.
def sign_bytes(y_sub: np.ndarray) -> np.ndarray:
    """y_sub [n][8] -> uint8 [n]"""
    neg = (np.asarray(y_sub) < 0).astype(np.uint8)
    return (neg << np.arange(8, dtype=np.uint8)).sum(axis=1).astype(np.uint8)


def signed_codewords(idx: np.ndarray, sgn: np.ndarray, codebook: np.ndarray) -> np.ndarray:
    """C[idx] with the sign bits applied: [n][8]"""
    c = np.asarray(codebook, dtype=F64)
    neg = (sgn.astype(np.int64)[:, None] >> np.arange(8)) & 1
    return np.where(neg == 1, -c[idx.astype(np.int64)], c[idx.astype(np.int64)])


def encode(x16: np.ndarray, codebook: np.ndarray, group_size: int = 0, start: int = 0,
           frozen_o: np.ndarray | None = None, given_b: np.ndarray | None = None,
           given_o: np.ndarray | None = None, return_debug: bool = False, sign_format: bool = False,
           rope_inv_freq=None, side_bits: int = 16):
    """Encode tokens [start, start+l) of one (sequence, kv-head, tensor) unit.

    x16       fp16 [l][d]
    codebook  [n_codes][sub]
    frozen_o  fp16 [n_groups][d]: append mode - use these stored means instead of
              computing new ones (a new token never forms a one-token group)
    given_b / given_o: override the stage-A results (two-stage parity protocol: the
              second stage is checked conditioned on the first stage's stored values)
    sign_format: codebook = 256 non-negative 8-dim magnitude codewords; codes are then
              u8 [l][2 d/8]: the d/8 indices followed by the d/8 sign bytes
    rope_inv_freq: [d/2] - x16 holds keys BEFORE the rotary embedding (Sec. 3.2): NSN runs on them
              as they are, v_nsn of token t is rotated by position start + t, then quantised;
              the stored mean o stays un-rotated
    side_bits: 4 = double quantization (Sec. 3.5).  s1 is rounded to fp16 and used for the first
              Normalize as always, but STORED as 4-bit codes per 64-token block (start must be a
              multiple of 64); the group means are stored as 4-bit codes per 32 channels and the
              Shift uses the dequantised mean; the stored per-token scale is a' = fp16(s2 alpha).
              The dict then holds the effective float64 values under the usual keys
              (a = b_hat a', b = b_hat, o = o_hat, so `dequantize` applies unchanged) and the stored
              fields a_stored, b_code, b_par, o_code, o_par (see quantize_side_info); given_o, if
              passed, is the dequantised mean array
    returns dict(codes u8 [l][d/sub], a fp16 [l], b fp16 [l], o fp16 [n_groups][d])
    """
    x = np.asarray(x16, dtype=F64)
    l, d = x.shape
    c = np.asarray(codebook, dtype=F64)
    sub = c.shape[1]
    assert d % sub == 0
    H = hadamard(d)

    # steps 1 and 2 (Normalize, Shift): the two stored side-information arrays b and o
    g = group_index(l, group_size, start)
    side = None
    if side_bits == 4:
        fixed_o = frozen_o if frozen_o is not None else given_o
        b16, o_raw = shift_stats(x16, group_size, start, given_b=given_b, raw_mean=True,
                                 given_o=None if fixed_o is None else np.zeros((1, d), dtype=np.float16))
        side = quantize_side_info(b16, np.zeros((1, d)) if fixed_o is not None else o_raw, start)
        o16 = side["o_hat"] if fixed_o is None else np.asarray(fixed_o, dtype=F64)
    else:
        assert side_bits == 16
        b16, o16 = shift_stats(x16, group_size, start, given_b=given_b,
                               given_o=frozen_o if frozen_o is not None else given_o)
    b = b16.astype(F64)
    n = _safe_div(x, b[:, None])
    o = np.asarray(o16, dtype=F64)
    ns = n - o[g]

    # step 3 (Normalize)
    s2 = token_scale(ns)
    vnsn = _safe_div(ns, s2[:, None])

    if rope_inv_freq is not None:
        vnsn = rope(vnsn, start + np.arange(l), rope_inv_freq)

    # Hadamard rotation (dense mat-vec), then Eq. (1) on contiguous sub-vectors
    y = vnsn @ H.T
    if sign_format:
        assert sub == 8 and np.all(c >= 0)
        ys = y.reshape(-1, sub)
        idx, best, second = nearest_codeword(np.abs(ys), c)
        sgn = sign_bytes(ys)
        yq = signed_codewords(idx, sgn, c).reshape(l, d)
        codes = np.concatenate([idx.reshape(l, d // sub), sgn.reshape(l, d // sub)], axis=1)
    else:
        codes, best, second = nearest_codeword(y.reshape(-1, sub), c)
        yq = c[codes].reshape(l, d)
        codes = codes.reshape(l, d // sub)

    # scale adjustment folded into the stored scale: a = s1 s2 alpha
    alpha = scale_adjust(y, yq)
    if side is not None:
        a_stored = fp16_rne(s2 * alpha)
        out = dict(codes=codes.astype(np.uint8), a=side["b_hat"] * a_stored.astype(F64), b=side["b_hat"], o=o,
                   a_stored=a_stored, b16=b16, b_code=side["b_code"], b_par=side["b_par"], o_code=side["o_code"],
                   o_par=side["o_par"])
    else:
        a16 = fp16_rne(b * s2 * alpha)
        out = dict(codes=codes.astype(np.uint8), a=a16, b=b16, o=o16)
    if return_debug:
        out.update(y=y, s2=s2, alpha=alpha, best=best.reshape(l, -1), second=second.reshape(l, -1), vnsn=vnsn)
    return out


def dequantize(codes, a16, b16, o16, codebook, group_size: int = 0, start: int = 0,
               sign_format: bool = False, rope_inv_freq=None) -> np.ndarray:
    """x_hat_t = b_t o_g + a_t H^T y_Q,t  (restore identity of Sec. 3.2 with s2 alpha in a).
    With rope_inv_freq (keys coded before the rotary embedding) the result is the key AFTER it:
    the mean enters as RoPE_t(o_g) (App. B, second line of the derivation)."""
    c = np.asarray(codebook, dtype=F64)
    l, J = codes.shape
    if sign_format:
        J //= 2
        d = J * c.shape[1]
        yq = signed_codewords(codes[:, :J].reshape(-1), codes[:, J:].reshape(-1), c).reshape(l, d)
    else:
        d = J * c.shape[1]
        yq = c[codes.astype(np.int64)].reshape(l, d)
    H = hadamard(d)
    g = group_index(l, group_size, start)
    a = np.asarray(a16, dtype=F64)
    b = np.asarray(b16, dtype=F64)
    o = np.asarray(o16, dtype=F64)
    mean_part = o[g]
    if rope_inv_freq is not None:
        mean_part = rope(mean_part, start + np.arange(l), rope_inv_freq)
    return b[:, None] * mean_part + a[:, None] * (yq @ H)  # H^T = H^-1; row form: yq @ H


# ----------------------------------------------------------------------------
# Decode attention over a coded cache (App. B; keys are taken as given unless rope_inv_freq is passed)
# ----------------------------------------------------------------------------
def decode_attention(q, kc: dict, vc: dict, codebook, softmax_scale: float,
                     group_size: int = 0, sign_format: bool = False, rope_inv_freq=None) -> np.ndarray:
    """out = softmax(scale * q K_hat^T) V_hat for q [r][d] (r query heads on one kv head).
    rope_inv_freq: the key cache was coded before the rotary embedding; q is the query after it."""
    q = np.atleast_2d(np.asarray(q, dtype=F64))
    k_hat = dequantize(kc["codes"], kc["a"], kc["b"], kc["o"], codebook, group_size, sign_format=sign_format,
                       rope_inv_freq=rope_inv_freq)
    v_hat = dequantize(vc["codes"], vc["a"], vc["b"], vc["o"], codebook, group_size, sign_format=sign_format)
    s = softmax_scale * (q @ k_hat.T)
    s = s - s.max(axis=1, keepdims=True)
    p = np.exp(s)
    p = p / p.sum(axis=1, keepdims=True)
    return p @ v_hat


def lut_scores(q, kc: dict, codebook, softmax_scale: float, group_size: int = 0) -> np.ndarray:
    """App. B last line: s1 s2 q_Had . v_Q + s1 q . o, evaluated through a per-sub-vector
    query x codebook table.  Independent of `dequantize`; must agree with q . K_hat."""
    q = np.atleast_2d(np.asarray(q, dtype=F64))
    c = np.asarray(codebook, dtype=F64)
    codes = kc["codes"].astype(np.int64)
    l, J = codes.shape
    sub = c.shape[1]
    H = hadamard(J * sub)
    q_had = q @ H.T
    g = group_index(l, group_size)
    out = np.zeros((q.shape[0], l), dtype=F64)
    a = np.asarray(kc["a"], dtype=F64)
    b = np.asarray(kc["b"], dtype=F64)
    o = np.asarray(kc["o"], dtype=F64)
    for r in range(q.shape[0]):
        lut = q_had[r].reshape(J, sub) @ c.T            # [J][n_codes]
        gathered = lut[np.arange(J)[None, :], codes].sum(axis=1)
        q_o = o @ q[r]                                   # [n_groups]
        out[r] = softmax_scale * (a * gathered + b * q_o[g])
    return out


def two_branch_scores_rope(q, kc: dict, codebook, softmax_scale: float, inv_freq, group_size: int = 0) -> np.ndarray:
    """App. B's last line for keys coded before the rotary embedding:
    s1 s2 q_Had . v_Q + s1 q . RoPE_t(o), the second branch evaluated as RoPE_{-t}(q) . o (the
    rotation is orthogonal, so it can be taken off the mean and put on the query with the
    opposite angle).  Independent of `dequantize`; must agree with q . K_hat."""
    q = np.atleast_2d(np.asarray(q, dtype=F64))
    c = np.asarray(codebook, dtype=F64)
    codes = kc["codes"].astype(np.int64)
    l, J = codes.shape
    H = hadamard(J * c.shape[1])
    q_had = q @ H.T
    g = group_index(l, group_size)
    a = np.asarray(kc["a"], dtype=F64)
    b = np.asarray(kc["b"], dtype=F64)
    o = np.asarray(kc["o"], dtype=F64)
    out = np.zeros((q.shape[0], l), dtype=F64)
    for r in range(q.shape[0]):
        for t in range(l):
            first = float(q_had[r] @ c[codes[t]].reshape(-1))
            q_back = rope(q[r][None, :], [-t], inv_freq)[0]
            out[r, t] = softmax_scale * (a[t] * first + b[t] * float(q_back @ o[g[t]]))
    return out


# ----------------------------------------------------------------------------
# Codebook: K-Means on standard normal data (Sec. 3.4, the K-Means baseline)
# ----------------------------------------------------------------------------
def build_codebook(samples: np.ndarray, n_codes: int = 256, iters: int = 50):
    """Lloyd iterations; init = first n_codes samples; empty cluster keeps its centroid.

    Returns (codebook float64 [n_codes][sub] rounded to fp16-representable values,
             inertia per-dimension MSE measured at the assignment of every iteration,
             final per-dimension MSE of the rounded codebook).
    """
    x = np.asarray(samples, dtype=F64)
    n, sub = x.shape
    c = x[:n_codes].copy()
    history = []
    for _ in range(iters):
        idx, best, _ = nearest_codeword(x, c)
        history.append(best.sum() / (n * sub))
        for k in range(n_codes):
            m = idx == k
            if m.any():
                c[k] = x[m].mean(axis=0)
    c = fp16_rne(c).astype(F64)
    _, best, _ = nearest_codeword(x, c)
    return c, np.asarray(history), best.sum() / (n * sub)


# ----------------------------------------------------------------------------
# Codebook fine-tuning (Sec. 3.4): lower the cosine distance between a standard-normal vector and
# its quantised version; the lookup is not differentiated, so a sample's gradient reaches only the
# centroid it was assigned to.  The paper gives no optimiser, rate or step count: plain full-batch
# gradient steps with a caller-chosen rate are this build's reading (parity with the paper's tuned
# codebook is unpinned; the gradient itself is pinned by finite differences in the tests).
# ----------------------------------------------------------------------------
def cosine_loss(samples, codebook, assignment=None) -> float:
    """mean over samples of 1 - cos(x, C[k(x)]); k = Eq. 1's nearest codeword unless given.
    Zero samples and zero codewords count as cosine 0."""
    x = np.asarray(samples, dtype=F64)
    c = np.asarray(codebook, dtype=F64)
    if assignment is None:
        assignment, _, _ = nearest_codeword(x, c)
    cq = c[assignment]
    den = np.linalg.norm(x, axis=1) * np.linalg.norm(cq, axis=1)
    cos = np.divide(np.sum(x * cq, axis=1), den, out=np.zeros_like(den), where=den > 0)
    return float(1.0 - cos.mean())


def cosine_loss_gradient(samples, codebook, assignment) -> np.ndarray:
    """d cosine_loss / d codebook for a fixed assignment:
    row k = -(1 / (N |c_k|)) * (S_k - (S_k . c_k^) c_k^),  S_k = sum of x / |x| over the samples of k."""
    x = np.asarray(samples, dtype=F64)
    c = np.asarray(codebook, dtype=F64)
    n = x.shape[0]
    nx = np.linalg.norm(x, axis=1, keepdims=True)
    xh = np.divide(x, nx, out=np.zeros_like(x), where=nx > 0)
    g = np.zeros_like(c)
    for k in range(c.shape[0]):
        m = assignment == k
        cn = float(np.linalg.norm(c[k]))
        if not m.any() or cn == 0.0:
            continue
        s_k = xh[m].sum(axis=0)
        ch = c[k] / cn
        g[k] = -(s_k - float(s_k @ ch) * ch) / (n * cn)
    return g


def finetune_codebook(samples, codebook, iters: int, lr: float):
    """`iters` steps of: assign by Eq. 1, C <- C - lr * gradient.  The result is rounded to fp16 once.
    Returns (codebook, mean cosine similarity before every step, mean cosine similarity of the result)."""
    x = np.asarray(samples, dtype=F64)
    c = np.asarray(codebook, dtype=F64).copy()
    history = []
    for _ in range(iters):
        idx, _, _ = nearest_codeword(x, c)
        history.append(1.0 - cosine_loss(x, c, idx))
        c = c - lr * cosine_loss_gradient(x, c, idx)
    c = fp16_rne(c).astype(F64)
    return c, np.asarray(history), 1.0 - cosine_loss(x, c)


# ----------------------------------------------------------------------------
# Storage accounting (Table 11, "Baseline" row: fp16 side information, no double quantisation)
# ----------------------------------------------------------------------------
def avg_bits(code_bits_per_dim: float, head_dim: int, group_size: int) -> float:
    """Bits per cached element: codes + two fp16 scales per token + one fp16 mean vector
    per group of `group_size` tokens."""
    scales = 2 * 16 / head_dim
    means = 16 * head_dim / (group_size * head_dim)
    return code_bits_per_dim + scales + means


def avg_bits_dq(code_bits_per_dim: float, head_dim: int, group_size: int, mean_dq: bool, scale_dq: bool) -> float:
    """Table 11's rows: means as 4-bit codes + (min, step) fp16 per 32 channels; s1 as 4-bit codes +
    (min, step) fp16 per `group_size` tokens next to the fp16 s2."""
    means = (4 * head_dim + (head_dim // 32) * 32) / (group_size * head_dim) if mean_dq else 16 / group_size
    scales = (16 + 4 + 32 / group_size) / head_dim if scale_dq else 2 * 16 / head_dim
    return code_bits_per_dim + scales + means


# ----------------------------------------------------------------------------
# Decode attention with the full-precision residual (Sec. 3.2 "Residual"): the most recent
# tokens are still fp16 and take part in the same softmax as the coded tokens
# ----------------------------------------------------------------------------
def decode_attention_residual(q, kc: dict, vc: dict, k_res16, v_res16, codebook, softmax_scale: float,
                              group_size: int = 0, sign_format: bool = False, rope_inv_freq=None) -> np.ndarray:
    """out = softmax(scale * q [K_hat ; K_res]^T) [V_hat ; V_res]; the coded part may be empty.
    rope_inv_freq: the coded keys were normalised before the rotary embedding; k_res16 holds the
    residual keys AFTER it (as attention uses them)."""
    q = np.atleast_2d(np.asarray(q, dtype=F64))
    k_res = np.asarray(k_res16, dtype=F64).reshape(-1, q.shape[1])
    v_res = np.asarray(v_res16, dtype=F64).reshape(-1, q.shape[1])
    if kc["codes"].shape[0] > 0:
        k_hat = dequantize(kc["codes"], kc["a"], kc["b"], kc["o"], codebook, group_size, sign_format=sign_format,
                           rope_inv_freq=rope_inv_freq)
        v_hat = dequantize(vc["codes"], vc["a"], vc["b"], vc["o"], codebook, group_size, sign_format=sign_format)
        k_all = np.concatenate([k_hat, k_res], axis=0)
        v_all = np.concatenate([v_hat, v_res], axis=0)
    else:
        k_all, v_all = k_res, v_res
    s = softmax_scale * (q @ k_all.T)
    s = s - s.max(axis=1, keepdims=True)
    p = np.exp(s)
    p = p / p.sum(axis=1, keepdims=True)
    return p @ v_all
