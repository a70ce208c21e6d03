"""CPU oracle for convolution with algorithm-based error detection (ABED).

TEST INFRASTRUCTURE ONLY.  Only tests/, __graft_entry__.smoke() and the
benchmark's cpu_baseline leg may import this module; the product path (the HIP
library and its Python binding) never does, and shares no code with it.

What is computed, each step following the paper:

* the convolution itself: Sec. 2.2, seven plain loops in C (conv_oracle.c);
* FC, the filter-checksum scheme, Sec. 3.1: wsum = sum_k w[k]; the extra output
  fmap conv(x, wsum) is compared element-wise with sum_k y[.,k];
* IC option 1, the batch-checksum scheme, Sec. 3.2: xsum = sum_n x[n]; the
  extra batch entry conv(xsum, w) is compared element-wise with sum_n y[n];
* the corner, where both checksums meet (the classical row+column scheme the
  paper recalls in Sec. 2.1): conv(xsum, wsum) against sum_n of the FC fmap
  and against sum_k of the IC fmap;
* overflow-free int8 checksums, Sec. 4.1: checksums are generated in int32 and
  stored as up to four int8 "digit" tensors; the extra fmaps of the digits are
  shifted left by 0, 8, 16, 24 and added.  (The paper prints the first shift
  as 1; with it the digits would not recombine to the checksum, so 0 is read.)
  Digits are balanced signed base-256, d in [-128,127]; any digit set with
  sum_i 256^i d_i = s is equally valid, only the recombined value is compared;
* reductions mod 2^32: the paper reduces in up to 64 bits and names modular
  arithmetic as the fallback (end of Sec. 4.1); all comparisons here are made
  on values reduced mod 2^32, and the exact int64 values are kept beside them;
* the epilog of Sec. 4.3 (scale in fp32, add bias, activation, clamp to int8)
  and the next layer's batch checksum taken from the epilog's output;
* FIC, the filter and input fmap checksum scheme, Sec. 3.3: the input is reduced
  to a checksum of the size of one filter, its dot product with the filter
  checksum (int64) must equal the sum of all outputs (int64);
* IC option 2 (Sec. 3.2): that same input checksum convolved with the K filters gives
  K values, which the outputs reduced over batch, height and width must equal;
* fp16 (Sec. 7): double-precision reference, checksums stored as a hi/lo pair
  of fp16 tensors, comparison against a threshold.

Parity pins for every function here are in tests/test_oracle_*.py.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None


def build(force=False):
    """Compile conv_oracle.c with gcc into oracle/liboracle_conv.so."""
    src = os.path.join(_HERE, "conv_oracle.c")
    out = os.path.join(_HERE, "liboracle_conv.so")
    if force or not os.path.exists(out) or os.path.getmtime(out) < os.path.getmtime(src):
        subprocess.check_call(["gcc", "-O3", "-march=x86-64-v3", "-fopenmp", "-shared", "-fPIC",
                               "-o", out, src])
    return out


def _lib():
    global _LIB
    if _LIB is None:
        _LIB = ctypes.CDLL(build())
        _LIB.oracle_num_threads.restype = ctypes.c_int
    return _LIB


def num_threads():
    return int(_lib().oracle_num_threads())


def _geom(shape):
    return [ctypes.c_int(int(v)) for v in (shape.N, shape.H, shape.W, shape.C, shape.K, shape.R, shape.S,
                                           shape.stride_h, shape.stride_w, shape.pad_h, shape.pad_w)]


def _ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p)


# ----------------------------------------------------------------------------
# Convolution (Sec. 2.2)
# ----------------------------------------------------------------------------
def conv_int(x, w, shape):
    """Exact integer convolution: x[N,H,W,C], w[K,R,S,C] (any integer dtype whose
    values fit int32) -> int64 y[N,P,Q,K].  N and K are taken from the arrays so
    that checksum tensors (one image, one filter) go through the same loops."""
    x32 = np.ascontiguousarray(x, dtype=np.int32)
    w32 = np.ascontiguousarray(w, dtype=np.int32)
    n, k = x32.shape[0], w32.shape[0]
    assert x32.shape[1:] == (shape.H, shape.W, shape.C) and w32.shape[1:] == (shape.R, shape.S, shape.C)
    y = np.empty((n, shape.P, shape.Q, k), dtype=np.int64)
    g = _geom(shape)
    g[0], g[4] = ctypes.c_int(n), ctypes.c_int(k)
    _lib().oracle_conv_i32(_ptr(x32), _ptr(w32), _ptr(y), *g)
    return y


def conv_int_points(x, w, shape, pts):
    """Exact values of the output elements pts[:,0..3] = (n,p,q,k) only."""
    x32 = np.ascontiguousarray(x, dtype=np.int32)
    w32 = np.ascontiguousarray(w, dtype=np.int32)
    pts = np.asarray(pts, dtype=np.int32)
    cols = [np.ascontiguousarray(pts[:, i]) for i in range(4)]
    y = np.empty(len(pts), dtype=np.int64)
    _lib().oracle_conv_i32_points(_ptr(x32), _ptr(w32), _ptr(y), ctypes.c_int(len(pts)),
                                  *[_ptr(c) for c in cols], *_geom(shape))
    return y


def conv_f64(x, w, shape):
    """Double-precision convolution of (fp16-valued) tensors -> float64 y[N,P,Q,K]."""
    xd = np.ascontiguousarray(x, dtype=np.float64)
    wd = np.ascontiguousarray(w, dtype=np.float64)
    n, k = xd.shape[0], wd.shape[0]
    y = np.empty((n, shape.P, shape.Q, k), dtype=np.float64)
    g = _geom(shape)
    g[0], g[4] = ctypes.c_int(n), ctypes.c_int(k)
    _lib().oracle_conv_f64(_ptr(xd), _ptr(wd), _ptr(y), *g)
    return y


def wrap32(a):
    """Reduce integers mod 2^32 and read them as two's-complement int32."""
    return (np.asarray(a, dtype=np.int64) & 0xFFFFFFFF).astype(np.uint32).view(np.int32)


# ----------------------------------------------------------------------------
# Checksum generation (Sec. 3.1, Sec. 3.2 option 1) and int8 digits (Sec. 4.1)
# ----------------------------------------------------------------------------
def filter_checksum(w):
    """wsum[r,s,c] = sum_k w[k,r,s,c]  (Sec. 3.1), exact in int64."""
    return np.asarray(w, dtype=np.int64).sum(axis=0)


def batch_checksum(x):
    """xsum[h,w,c] = sum_n x[n,h,w,c]  (Sec. 3.2, option 1), exact in int64."""
    return np.asarray(x, dtype=np.int64).sum(axis=0)


def num_digits_for_count(count):
    """Digits that always suffice for a sum of `count` int8 values: the sum lies
    in [-128*count, 127*count] (8 + log2(count) bits, Sec. 4.1) and d balanced
    base-256 digits cover [-128*(256^d-1)/255, 127*(256^d-1)/255]."""
    d = 1
    while 128 * count > 128 * (256 ** d - 1) // 255:
        d += 1
    return d


def split_digits(s, ndigits):
    """Balanced signed base-256 digits of integer array s: returns int8
    d[ndigits, ...] with sum_i 256^i d[i] == s; raises if ndigits is too few."""
    rest = np.asarray(s, dtype=np.int64).copy()
    out = np.empty((ndigits,) + rest.shape, dtype=np.int8)
    for i in range(ndigits):
        d = ((rest + 128) % 256) - 128          # in [-128, 127], congruent to rest mod 256
        out[i] = d.astype(np.int8)
        rest = (rest - d) // 256                # exact division
    if np.any(rest != 0):
        raise OverflowError("checksum does not fit %d int8 digits" % ndigits)
    return out


def recombine_digits(parts):
    """sum_i parts[i] << (8 i), exact in int64 (parts: sequence of integer arrays)."""
    tot = np.zeros_like(np.asarray(parts[0], dtype=np.int64))
    for i, p in enumerate(parts):
        tot = tot + (np.asarray(p, dtype=np.int64) << (8 * i))
    return tot


def flip_bit(arr, flat_index, bit):
    """Flip one bit of one element of an integer/fp16 array, in place, through its raw bits."""
    a = arr.reshape(-1)
    u = a.view({1: np.uint8, 2: np.uint16, 4: np.uint32, 8: np.uint64}[a.dtype.itemsize])
    u[flat_index] ^= u.dtype.type(1 << bit)


# ----------------------------------------------------------------------------
# Epilog (Sec. 4.3) and the next layer's batch checksum
# ----------------------------------------------------------------------------
def epilog_int8(acc32, scale, bias, relu):
    """ConvOut (int32) -> int8: convert to fp32, multiply by the per-channel
    scale, add the per-channel bias (two separately rounded fp32 operations),
    apply ReLU, round to nearest even, clamp to [-128, 127]."""
    t = np.asarray(acc32, dtype=np.int32).astype(np.float32)
    t = (t * np.asarray(scale, dtype=np.float32)).astype(np.float32)
    t = (t + np.asarray(bias, dtype=np.float32)).astype(np.float32)
    if relu:
        t = np.maximum(t, np.float32(0.0))
    q = np.rint(t)
    q = np.clip(q, -128.0, 127.0)
    return q.astype(np.int8)


# ----------------------------------------------------------------------------
# The whole checked convolution, int8
# ----------------------------------------------------------------------------
def abed_int8(x, w, shape, wchk=None, xchk=None, acc_flip=None, stored_flip=None,
              check_sees_stored=False, epilog=None):
    """Checked int8 convolution.

    x int8[N,H,W,C], w int8[K,R,S,C].  wchk int8[d_f,R,S,C] / xchk int8[d_i,H,W,C]
    are the digit tensors of the filter / batch checksum; when None they are
    generated from w / x here (a test passes its own to model a checksum that
    was made before x or w was corrupted, or a corrupted checksum).
    acc_flip = (flat index into y[N,P,Q,K], bit): one accumulator bit flipped
    after the convolution and before both the reductions and the store.
    stored_flip = same, applied to the stored ConvOut only; the reductions see
    it only if check_sees_stored (the variants that verify by reading ConvOut
    back from memory: Sec. 4.3, unfused option).
    epilog = (scale[K], bias[K], relu) or None.

    Returns a dict; every *_bad map is boolean:
      y        int32[N,P,Q,K]  ConvOut as stored
      yf       int32[N,P,Q]    extra fmap of the checksum filter, mod 2^32
      yi       int32[P,Q,K]    extra batch entry of the checksum image, mod 2^32
      yfi      int32[P,Q]      conv(xsum, wsum), mod 2^32
      rs, cs   int32           sum_k y, sum_n y, mod 2^32
      fc_bad[N,P,Q] = rs != yf;  ic_bad[P,Q,K] = cs != yi
      corner_bad[P,Q] = (sum_n yf != yfi) or (sum_k yi != yfi)
      out8, xsum_next, xchk_next when an epilog is given.
    """
    N, K = shape.N, shape.K
    x = np.asarray(x, dtype=np.int8)
    w = np.asarray(w, dtype=np.int8)
    if wchk is None:
        wchk = split_digits(filter_checksum(w), num_digits_for_count(K))
    if xchk is None:
        xchk = split_digits(batch_checksum(x), num_digits_for_count(N))

    y64 = conv_int(x, w, shape)                       # exact
    y_checked = wrap32(y64).copy()
    if acc_flip is not None:
        flip_bit(y_checked, *acc_flip)
    y_stored = y_checked.copy()
    if stored_flip is not None:
        flip_bit(y_stored, *stored_flip)
        if check_sees_stored:
            y_checked = y_stored

    # extra fmaps, one per digit, recombined by shifts (Sec. 4.1)
    yf_digits = conv_int(x, wchk, shape)              # [N,P,Q,d_f]
    yf = wrap32(recombine_digits([yf_digits[..., i] for i in range(wchk.shape[0])]))
    yi_digits = conv_int(xchk, w, shape)              # [d_i,P,Q,K]
    yi = wrap32(recombine_digits([yi_digits[j] for j in range(xchk.shape[0])]))
    yfi_digits = conv_int(xchk, wchk, shape)          # [d_i,P,Q,d_f]
    yfi = wrap32(recombine_digits(
        [recombine_digits([yfi_digits[j, :, :, i] for i in range(wchk.shape[0])])
         for j in range(xchk.shape[0])]))

    yc = y_checked.astype(np.int64)
    rs = wrap32(yc.sum(axis=3))                       # over k  (Sec. 3.1)
    cs = wrap32(yc.sum(axis=0))                       # over n  (Sec. 3.2)
    res = dict(y=y_stored, y_exact=y64, yf=yf, yi=yi, yfi=yfi, rs=rs, cs=cs, wchk=wchk, xchk=xchk)
    res["fc_bad"] = rs != yf
    res["ic_bad"] = cs != yi
    res["corner_bad"] = ((wrap32(yf.astype(np.int64).sum(axis=0)) != yfi)
                         | (wrap32(yi.astype(np.int64).sum(axis=2)) != yfi))
    if epilog is not None:
        scale, bias, relu = epilog
        out8 = epilog_int8(y_stored, scale, bias, relu)
        res["out8"] = out8
        res["xsum_next"] = batch_checksum(out8)       # [P,Q,K], the next layer's IC input
        res["xchk_next"] = split_digits(res["xsum_next"], num_digits_for_count(N))
    return res


# ----------------------------------------------------------------------------
# FIC, the filter and input fmap checksum scheme (Sec. 3.3)
# ----------------------------------------------------------------------------
def patch_checksum(x, shape):
    """Input fmap checksum of the FIC scheme (Sec. 3.2 option 2, used by Sec. 3.3): a
    tensor of the size of one filter, X[r,s,c] = sum over the batch and over all
    output positions (p,q) of the input element that filter element (r,s,c) meets
    there, zero where the window hangs over the padding.  Exact, int64[R,S,C];
    each entry is a sum of N*P*Q int8 values (8 + log2(PQN) bits, Sec. 4.1).

    x may also be the batch-summed image sum_n x[n] (three axes [H,W,C], any integer
    type): the previous layer's fused kernel can emit that sum of its own output
    (Sec. 4.3, the option that generates the next layer's input checksum), and the
    checksum is linear in x."""
    sh = shape
    x = np.asarray(x)
    if x.ndim == 3:
        x = x[None].astype(np.int64)
    else:
        x = x.astype(np.int8)
    xp = np.zeros((x.shape[0], sh.H + 2 * sh.pad_h, sh.W + 2 * sh.pad_w, sh.C), dtype=np.int64)
    xp[:, sh.pad_h:sh.pad_h + sh.H, sh.pad_w:sh.pad_w + sh.W] = x
    X = np.zeros((sh.R, sh.S, sh.C), dtype=np.int64)
    for r in range(sh.R):
        for s_ in range(sh.S):
            for p in range(sh.P):
                for q in range(sh.Q):
                    X[r, s_] += xp[:, p * sh.stride_h + r, q * sh.stride_w + s_].sum(axis=0)
    return X


def abed_fic_int8(x, w, shape, wsum=None, xpatch=None, acc_flip=None, epilog=None):
    """FIC check of an int8 convolution (Sec. 3.3; widths of Sec. 4.1; tasks of Sec. 4.3).

    The filter checksum wsum[r,s,c] = sum_k w[k] (int32 suffices) and the input
    checksum X[r,s,c] (patch_checksum; int32 suffices) meet in a dot product over
    C*R*S elements, an int64; the convolution output is reduced to one int64;
    the two must be equal.  wsum / xpatch may be passed in to model checksums
    made before w or x was corrupted.  acc_flip = (flat index into y, bit): one
    accumulator bit flipped before the reduction and the store.

    Returns dict: y int32[N,P,Q,K] as stored, ocs (output checksum) and dot as
    Python ints, bad = ocs != dot, wsum, xpatch, out8 when an epilog is given."""
    x = np.asarray(x, dtype=np.int8)
    w = np.asarray(w, dtype=np.int8)
    if wsum is None:
        wsum = filter_checksum(w)
    if xpatch is None:
        xpatch = patch_checksum(x, shape)
    y = wrap32(conv_int(x, w, shape)).copy()
    if acc_flip is not None:
        flip_bit(y, *acc_flip)
    ocs = int(y.astype(np.int64).sum())
    dot = int((np.asarray(xpatch, dtype=np.int64) * np.asarray(wsum, dtype=np.int64)).sum())
    res = dict(y=y, ocs=ocs, dot=dot, bad=ocs != dot, wsum=np.asarray(wsum), xpatch=np.asarray(xpatch))
    if epilog is not None:
        scale, bias, relu = epilog
        res["out8"] = epilog_int8(y, scale, bias, relu)
        # what the next layer's input checksum is made from when this layer's kernel emits it
        # (Sec. 4.3): the batch sum of the epilog's output
        res["xsum_next"] = batch_checksum(res["out8"])
    return res


def abed_ic2_int8(x, w, shape, xpatch=None, acc_flip=None, epilog=None):
    """IC option 2 of Sec. 3.2: the input fmaps are reduced to a checksum tensor of the
    size of one filter (patch_checksum), that tensor is convolved with the K filters,
    which gives exactly K values, and the output fmaps, reduced over height, width and
    batch, must equal those K values element by element.  Sums are exact (int64,
    widths of Sec. 4.1).  xpatch may be passed in to model a checksum made before x was
    corrupted; acc_flip as in abed_fic_int8.

    Returns dict: y int32[N,P,Q,K] as stored, osum int64[K] (reduced outputs), chk
    int64[K] (checksum tensor convolved with the filters), bad bool[K] = osum != chk,
    xpatch, out8 when an epilog is given."""
    x = np.asarray(x, dtype=np.int8)
    w = np.asarray(w, dtype=np.int8)
    if xpatch is None:
        xpatch = patch_checksum(x, shape)
    y = wrap32(conv_int(x, w, shape)).copy()
    if acc_flip is not None:
        flip_bit(y, *acc_flip)
    osum = y.astype(np.int64).sum(axis=(0, 1, 2))
    # the checksum tensor has the extent of one filter, so its convolution with filter k
    # has a single output position: the sum of the element-wise products
    X = np.asarray(xpatch, dtype=np.int64)
    chk = np.array([int((X * w[k].astype(np.int64)).sum()) for k in range(shape.K)], dtype=np.int64)
    res = dict(y=y, osum=osum, chk=chk, bad=osum != chk, xpatch=np.asarray(xpatch))
    if epilog is not None:
        scale, bias, relu = epilog
        res["out8"] = epilog_int8(y, scale, bias, relu)
    return res


# ----------------------------------------------------------------------------
# fp16 (Sec. 7)
# ----------------------------------------------------------------------------
def split_hi_lo(s):
    """A high-precision checksum stored as two fp16 tensors: hi = fp16(s),
    lo = fp16(s - hi)  ("multiple fp16 values", Sec. 7)."""
    s = np.asarray(s, dtype=np.float64)
    with np.errstate(invalid="ignore", over="ignore"):       # a non-finite sum stays non-finite in both parts
        hi = s.astype(np.float16)
        lo = (s - hi.astype(np.float64)).astype(np.float16)
    return np.stack([hi, lo])


def threshold_bad(s, c, rtol, atol, mag=None):
    """Mismatch test for floating point (Sec. 7: the two reduced values are "close enough" when they
    differ by no more than a threshold).  Two readings of the threshold's magnitude:

    mag is None: relative to the compared values, tol = rtol * max(|s|, |c|) + atol;
    mag given  : relative to the L1 norm of what was reduced, tol = rtol * mag + atol with
                 mag = sum of |y| over the elements that s sums (rounding error of a sum grows with
                 that norm, not with the sum, which may cancel to zero).

    A mismatch is  not (|s - c| <= tol); a NaN or an infinity on either side is a mismatch."""
    s = np.asarray(s, dtype=np.float64)
    c = np.asarray(c, dtype=np.float64)
    with np.errstate(invalid="ignore"):
        scale = np.maximum(np.abs(s), np.abs(c)) if mag is None else np.asarray(mag, dtype=np.float64)
        tol = rtol * scale + atol
        ok = (np.abs(s - c) <= tol) & np.isfinite(s) & np.isfinite(c) & np.isfinite(tol)
    return ~ok


def threshold_margin(s, c, rtol, atol, mag=None):
    """|s - c| - tol of threshold_bad (positive = mismatch), for guard bands around the decision."""
    s = np.asarray(s, dtype=np.float64)
    c = np.asarray(c, dtype=np.float64)
    with np.errstate(invalid="ignore"):
        scale = np.maximum(np.abs(s), np.abs(c)) if mag is None else np.asarray(mag, dtype=np.float64)
        return np.abs(s - c) - (rtol * scale + atol)


def abed_fp16(x, w, shape, rtol, atol, wchk=None, xchk=None, acc_flip=None, out_dtype=np.float16, l1=False):
    """Checked fp16 convolution, double-precision reference.

    The reductions are taken over the (double) accumulators before the output
    is rounded, as the fused kernels reduce their fp32 accumulators.  acc_flip =
    (flat index, bit 0..15) flips a bit of the value rounded to fp16, and the
    corrupted value replaces the accumulator in the reductions and in the store.
    l1 selects the threshold's magnitude (threshold_bad): the compared values, or the sum of |y| over
    the reduced elements (rs_abs over the filters for FC, cs_abs over the batch for IC; for the corner
    the same norms of the checksum fmaps).
    Returns y (out_dtype), yf, yi, yfi, rs, cs (float64), fc_bad, ic_bad,
    corner_bad, the signed margins  |s-c| - tol  of both checks, and xchk_next (the hi/lo batch checksum of
    the fp16 outputs, for the next layer)."""
    x = np.asarray(x, dtype=np.float16)
    w = np.asarray(w, dtype=np.float16)
    if wchk is None:
        wchk = split_hi_lo(np.asarray(w, dtype=np.float64).sum(axis=0))
    if xchk is None:
        xchk = split_hi_lo(np.asarray(x, dtype=np.float64).sum(axis=0))
    y = conv_f64(x, w, shape)
    if acc_flip is not None:
        idx, bit = acc_flip
        v = np.array([y.reshape(-1)[idx]], dtype=np.float16)
        flip_bit(v, 0, bit)
        y.reshape(-1)[idx] = np.float64(v[0])
    yf = conv_f64(x, wchk, shape).sum(axis=3)                  # hi + lo
    yi = conv_f64(xchk, w, shape).sum(axis=0)
    yfi = conv_f64(xchk, wchk, shape).sum(axis=(0, 3))
    rs, cs = y.sum(axis=3), y.sum(axis=0)
    rs_abs, cs_abs = np.abs(y).sum(axis=3), np.abs(y).sum(axis=0)

    res = dict(y=y.astype(out_dtype), y_exact=y, yf=yf, yi=yi, yfi=yfi, rs=rs, cs=cs, rs_abs=rs_abs, cs_abs=cs_abs,
               wchk=wchk, xchk=xchk)
    # the next layer's batch checksum, generated with the output (Sec. 4.3, the option that also generates the next
    # layer's input checksum): the sum over the batch of the values the next layer will read, i.e. of the outputs
    # rounded to fp16, stored as a hi/lo pair like every fp16 checksum (Sec. 7)
    res["xchk_next"] = split_hi_lo(y.astype(np.float16).astype(np.float64).sum(axis=0))
    res["fc_margin"] = threshold_margin(rs, yf, rtol, atol, rs_abs if l1 else None)
    res["ic_margin"] = threshold_margin(cs, yi, rtol, atol, cs_abs if l1 else None)
    res["fc_bad"] = threshold_bad(rs, yf, rtol, atol, rs_abs if l1 else None)
    res["ic_bad"] = threshold_bad(cs, yi, rtol, atol, cs_abs if l1 else None)
    res["corner_bad"] = (threshold_bad(yf.sum(axis=0), yfi, rtol, atol, np.abs(yf).sum(axis=0) if l1 else None)
                         | threshold_bad(yi.sum(axis=2), yfi, rtol, atol, np.abs(yi).sum(axis=2) if l1 else None))
    return res
