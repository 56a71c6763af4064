"""ctypes binding of the CPU oracle (oracle/dgq_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and
by bench.py's cpu_baseline leg.  The product package never imports it.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dgq_oracle.c")
_LIB = os.path.join(_HERE, "libdgq_oracle.so")
GRANULE = 64

_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no FMA contraction, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call([
            "gcc", "-O2", "-ffp-contract=off", "-fno-fast-math", "-std=c11",
            "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def lib():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_LIB)
        _lib.dgqo_two_means.restype = C.c_int64
    return _lib


def _p(a, t=None):
    if a is None:
        return None
    return a.ctypes.data_as(C.c_void_p)


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def two_means(v):
    """Returns (n_lower, tau, order)."""
    v = _f32(v)
    tau = C.c_float()
    order = np.empty(v.size, dtype=np.int64)
    k = lib().dgqo_two_means(_p(v), C.c_int64(v.size), C.byref(tau), _p(order))
    return int(k), np.float32(tau.value), order


@dataclass
class Groups:
    C: int
    act_bits: int
    G: int
    P: int
    NG: int
    Kp: int
    n_outlier_channels: int
    n_regular_groups: int
    dstar: int
    n_class1_rows: int
    perm: np.ndarray      # [Kp] int32, -1 = padding
    goff: np.ndarray      # [NG+1]
    glen: np.ndarray      # [NG]
    tau_pix: np.float32
    s: np.ndarray         # [2, NG]
    z: np.ndarray
    inv_s: np.ndarray
    D_channel: float
    D_pixel: float
    cal_row_class: np.ndarray
    taus: np.ndarray = None   # [P-1] ascending row-range thresholds (class = number below the range)
    mode: int = -1            # -1 hybrid grid; 0 / 1 single-dimension grouping along channel / pixel


def calibrate(x, act_bits: int, G: int, P: int = 2, granule: int = GRANULE) -> Groups:
    x = _f32(x)
    rows, Cc = x.shape
    ng_cap = 2 * ((Cc + G - 1) // G) + 2
    kp_cap = Cc + granule * ng_cap
    scal = np.zeros(8, dtype=np.int32)
    perm = np.full(kp_cap, -1, dtype=np.int32)
    goff = np.zeros(ng_cap + 1, dtype=np.int32)
    glen = np.zeros(ng_cap, dtype=np.int32)
    tau = C.c_float()
    s = np.zeros((2, ng_cap), dtype=np.float32)
    z = np.zeros((2, ng_cap), dtype=np.float32)
    inv_s = np.zeros((2, ng_cap), dtype=np.float32)
    D = np.zeros(2, dtype=np.float64)
    rc_cls = np.zeros(rows, dtype=np.uint8)
    rc = lib().dgqo_calibrate(_p(x), C.c_int64(rows), C.c_int32(Cc), C.c_int32(act_bits),
                              C.c_int32(G), C.c_int32(P), C.c_int32(granule),
                              C.c_int32(ng_cap), C.c_int32(kp_cap), _p(scal), _p(perm),
                              _p(goff), _p(glen), C.byref(tau), _p(s), _p(z), _p(inv_s),
                              _p(D), _p(rc_cls))
    if rc != 0:
        raise RuntimeError("oracle calibrate: capacity too small")
    ng, kp = int(scal[0]), int(scal[1])
    return Groups(C=Cc, act_bits=act_bits, G=G, P=P, NG=ng, Kp=kp,
                  n_outlier_channels=int(scal[2]), n_regular_groups=int(scal[3]),
                  dstar=int(scal[4]), n_class1_rows=int(scal[5]),
                  perm=perm[:kp].copy(), goff=goff[:ng + 1].copy(), glen=glen[:ng].copy(),
                  tau_pix=np.float32(tau.value),
                  s=np.ascontiguousarray(s[:, :ng]), z=np.ascontiguousarray(z[:, :ng]),
                  inv_s=np.ascontiguousarray(inv_s[:, :ng]),
                  D_channel=float(D[0]), D_pixel=float(D[1]), cal_row_class=rc_cls,
                  taus=np.array([tau.value], dtype=np.float32))


def im2col3x3(x, B: int, H: int, W: int):
    """The 3 x 3 neighbourhoods of a [B*H*W, C] activation map (pixels row-major, one row
    per pixel) as rows of 9 C values: tap t = 3 (dy + 1) + (dx + 1) holds the channels of
    pixel (h + dy, w + dx), zeros outside the image (stride 1, zero padding 1)."""
    x = np.asarray(x)
    Cc = x.shape[1]
    img = x.reshape(B, H, W, Cc)
    pad = np.zeros((B, H + 2, W + 2, Cc), dtype=x.dtype)
    pad[:, 1:H + 1, 1:W + 1] = img
    taps = [pad[:, 1 + dy:1 + dy + H, 1 + dx:1 + dx + W] for dy in (-1, 0, 1) for dx in (-1, 0, 1)]
    return np.concatenate(taps, axis=-1).reshape(B * H * W, 9 * Cc)


def groups_for_conv3x3(g: Groups) -> Groups:
    """The group tables of a 3 x 3 convolution over an input grouped by g (one pixel class):
    the unfolded input has 9 C channels, tap t's copy of channel c being channel t C + c, and
    every tap keeps the channel groups, scales and offsets of g."""
    assert g.P == 1
    T = 9
    perm = np.concatenate([np.where(g.perm >= 0, g.perm + t * g.C, -1) for t in range(T)]).astype(np.int32)
    goff = np.concatenate([g.goff[:-1] + t * g.Kp for t in range(T)] + [[T * g.Kp]]).astype(np.int32)
    return Groups(C=T * g.C, act_bits=g.act_bits, G=g.G, P=1, NG=T * g.NG, Kp=T * g.Kp,
                  n_outlier_channels=T * g.n_outlier_channels, n_regular_groups=T * g.n_regular_groups,
                  dstar=g.dstar, n_class1_rows=0, perm=perm, goff=goff,
                  glen=np.tile(g.glen, T).astype(np.int32), tau_pix=g.tau_pix,
                  s=np.ascontiguousarray(np.tile(g.s, (1, T))), z=np.ascontiguousarray(np.tile(g.z, (1, T))),
                  inv_s=np.ascontiguousarray(np.tile(g.inv_s, (1, T))),
                  D_channel=g.D_channel, D_pixel=g.D_pixel, cal_row_class=g.cal_row_class,
                  taus=g.taus, mode=g.mode)


def k_means(v, K: int):
    """Exact 1-D K-means.  Returns (k, bounds [k+1], taus [k-1], order)."""
    v = _f32(v)
    bounds = np.zeros(K + 1, dtype=np.int64)
    taus = np.zeros(max(K - 1, 1), dtype=np.float32)
    order = np.empty(v.size, dtype=np.int64)
    lib().dgqo_k_means.restype = C.c_int32
    k = int(lib().dgqo_k_means(_p(v), C.c_int64(v.size), C.c_int32(K), _p(bounds), _p(taus), _p(order)))
    return k, bounds[:k + 1].copy(), taus[:k - 1].copy(), order


def calibrate_kmeans(x, act_bits: int, K: int, dim: int = -1, granule: int = GRANULE) -> Groups:
    """Grouping along one dimension (dim -1: argmax D_d, 0: channel, 1: pixel) into K clusters."""
    x = _f32(x)
    rows, Cc = x.shape
    assert 1 <= K <= 16
    ng_cap = K
    kp_cap = Cc + granule * (K + 1)
    scal = np.zeros(8, dtype=np.int32)
    perm = np.full(kp_cap, -1, dtype=np.int32)
    goff = np.zeros(ng_cap + 1, dtype=np.int32)
    glen = np.zeros(ng_cap, dtype=np.int32)
    taus = np.zeros(64, dtype=np.float32)
    s = np.zeros((K, ng_cap), dtype=np.float32)
    z = np.zeros((K, ng_cap), dtype=np.float32)
    inv_s = np.zeros((K, ng_cap), dtype=np.float32)
    D = np.zeros(2, dtype=np.float64)
    rc_cls = np.zeros(rows, dtype=np.uint8)
    rc = lib().dgqo_calibrate_kmeans(_p(x), C.c_int64(rows), C.c_int32(Cc), C.c_int32(act_bits),
                                     C.c_int32(K), C.c_int32(dim), C.c_int32(granule),
                                     C.c_int32(ng_cap), C.c_int32(kp_cap), _p(scal), _p(perm),
                                     _p(goff), _p(glen), _p(taus), _p(s), _p(z), _p(inv_s),
                                     _p(D), _p(rc_cls))
    if rc != 0:
        raise RuntimeError("oracle calibrate_kmeans: capacity too small")
    ng, kp, P = int(scal[0]), int(scal[1]), int(scal[6])
    taus = taus[:P - 1].copy() if P > 1 else np.array([np.inf], dtype=np.float32)
    return Groups(C=Cc, act_bits=act_bits, G=0, P=P, NG=ng, Kp=kp, n_outlier_channels=0,
                  n_regular_groups=0, dstar=int(scal[4]), n_class1_rows=int(scal[5]),
                  perm=perm[:kp].copy(), goff=goff[:ng + 1].copy(), glen=glen[:ng].copy(),
                  tau_pix=np.float32(taus[0]),
                  s=np.ascontiguousarray(s[:P, :ng]), z=np.ascontiguousarray(z[:P, :ng]),
                  inv_s=np.ascontiguousarray(inv_s[:P, :ng]),
                  D_channel=float(D[0]), D_pixel=float(D[1]), cal_row_class=rc_cls,
                  taus=taus, mode=int(scal[7]))


def quantize_act(g: Groups, x, want_dq: bool = False):
    """Returns dict(q [rows,Kp] u8, cls [rows] u8, xdq [rows,C] f64, clip [rows,C] u8)."""
    x = _f32(x)
    rows = x.shape[0]
    assert x.shape[1] == g.C
    q = np.zeros((rows, g.Kp), dtype=np.uint8)
    cls = np.zeros(rows, dtype=np.uint8)
    xdq = np.zeros((rows, g.C), dtype=np.float64) if want_dq else None
    clip = np.zeros((rows, g.C), dtype=np.uint8) if want_dq else None
    taus = _f32(g.taus if g.taus is not None else [g.tau_pix])
    lib().dgqo_quantize_act_multi(_p(x), C.c_int64(rows), C.c_int32(g.C), C.c_int32(g.act_bits),
                                  C.c_int32(g.NG), C.c_int32(g.NG), _p(g.perm), _p(g.goff),
                                  _p(g.glen), _p(taus), C.c_int32(taus.size), _p(g.s), _p(g.z),
                                  _p(g.inv_s), _p(q), _p(cls), _p(xdq), _p(clip))
    return dict(q=q, cls=cls, xdq=xdq, clip=clip)


def quantize_weight(w, w_bits: int):
    w = _f32(w)
    O, Cc = w.shape
    wq = np.zeros((O, Cc), dtype=np.int8)
    sw = np.zeros(O, dtype=np.float32)
    lib().dgqo_quantize_weight(_p(w), C.c_int32(O), C.c_int32(Cc), C.c_int32(w_bits),
                               _p(wq), _p(sw))
    return wq, sw


def linear(g: Groups, q, cls, wq, sw, bias=None, want_acc: bool = False):
    """q [rows,Kp] u8, cls [rows] u8 -> (Y [rows,O] f32, acc [rows,O,NG] i32 or None)."""
    q = np.ascontiguousarray(q, dtype=np.uint8)
    cls = np.ascontiguousarray(cls, dtype=np.uint8)
    wq = np.ascontiguousarray(wq, dtype=np.int8)
    sw = _f32(sw)
    rows = q.shape[0]
    O = wq.shape[0]
    assert q.shape[1] == g.Kp and wq.shape[1] == g.C
    y = np.zeros((rows, O), dtype=np.float32)
    acc = np.zeros((rows, O, g.NG), dtype=np.int32) if want_acc else None
    b = _f32(bias) if bias is not None else None
    lib().dgqo_linear(_p(q), _p(cls), C.c_int64(rows), C.c_int32(g.C), C.c_int32(O),
                      C.c_int32(g.act_bits), C.c_int32(g.NG), C.c_int32(g.NG), _p(g.perm),
                      _p(g.goff), _p(g.glen), _p(g.s), _p(g.z), _p(wq), _p(sw), _p(b),
                      _p(y), _p(acc))
    return y, acc


def geglu(y):
    """y [rows, O] fp32 -> [rows, O/2]: first half times GELU(second half), in double."""
    y = _f32(y)
    rows, O = y.shape
    assert O % 2 == 0
    out = np.zeros((rows, O // 2), dtype=np.float32)
    lib().dgqo_geglu(_p(y), C.c_int64(rows), C.c_int32(O), _p(out))
    return out


def attn_probs(Q, K, key_bias=None):
    """Q [B,N,H,d], K [B,nk,H,d] -> A [B,H,N,nk] fp32."""
    Q = _f32(Q)
    K = _f32(K)
    B, N, H, d = Q.shape
    nk = K.shape[1]
    kb = _f32(key_bias) if key_bias is not None else None
    A = np.zeros((B, H, N, nk), dtype=np.float32)
    lib().dgqo_attn_probs(_p(Q), _p(K), _p(kb), C.c_int32(B), C.c_int32(N), C.c_int32(H),
                          C.c_int32(d), C.c_int32(nk), _p(A))
    return A


def xattn_logq(A, V, bits: int, want_ahat: bool = False, s_in=None):
    """A [B,H,N,nk] fp32, V [B,nk,H,d] -> dict(s, codes, margin, ahat, out [B,N,H,d])."""
    A = _f32(A)
    V = _f32(V)
    B, H, N, nk = A.shape
    d = V.shape[3]
    s = np.zeros(B, dtype=np.float32)
    codes = np.zeros((B, H, N, nk - 1), dtype=np.uint8)
    margin = np.zeros((B, H, N, nk - 1), dtype=np.float32)
    ahat = np.zeros((B, H, N, nk), dtype=np.float64) if want_ahat else None
    out = np.zeros((B, N, H, d), dtype=np.float32)
    if s_in is None:
        lib().dgqo_xattn_logq(_p(A), _p(V), C.c_int32(B), C.c_int32(N), C.c_int32(H),
                              C.c_int32(d), C.c_int32(nk), C.c_int32(bits), _p(s), _p(codes),
                              _p(margin), _p(ahat), _p(out))
    else:
        s_in = _f32(s_in)
        assert s_in.shape == (B,)
        lib().dgqo_xattn_logq_static(_p(A), _p(V), C.c_int32(B), C.c_int32(N), C.c_int32(H),
                                     C.c_int32(d), C.c_int32(nk), C.c_int32(bits), _p(s_in), _p(s),
                                     _p(codes), _p(margin), _p(ahat), _p(out))
    return dict(s=s, codes=codes, margin=margin, ahat=ahat, out=out)


def selfattn(Q, K, V, bits: int, s_in, want_ahat: bool = False):
    """Self-attention with every probability log2-quantized against the given scale
    s_in [B].  Q [B,Nq,H,d] (any subset of the queries), K, V [B,nk,H,d] ->
    dict(A, s (= max A per prompt), codes [B,H,Nq,nk], margin, ahat, out [B,Nq,H,d])."""
    A = attn_probs(Q, K, None)
    V = _f32(V)
    B, H, N, nk = A.shape
    d = V.shape[3]
    s_in = _f32(s_in)
    assert s_in.shape == (B,)
    s = np.zeros(B, dtype=np.float32)
    codes = np.zeros((B, H, N, nk), dtype=np.uint8)
    margin = np.zeros((B, H, N, nk), dtype=np.float32)
    ahat = np.zeros((B, H, N, nk), dtype=np.float64) if want_ahat else None
    out = np.zeros((B, N, H, d), dtype=np.float32)
    lib().dgqo_selfattn_logq(_p(A), _p(V), C.c_int32(B), C.c_int32(N), C.c_int32(H), C.c_int32(d),
                             C.c_int32(nk), C.c_int32(bits), _p(s_in), _p(s), _p(codes), _p(margin),
                             _p(ahat), _p(out))
    return dict(A=A, s=s, codes=codes, margin=margin, ahat=ahat, out=out)


def quantize_value(V, bits: int = 8):
    """V [B,nk,H,d] -> dict(vhat fp32 [B,nk,H,d], codes u8, params [B,H,2] = (s, z))."""
    V = _f32(V)
    B, nk, H, d = V.shape
    vhat = np.zeros_like(V)
    codes = np.zeros(V.shape, dtype=np.uint8)
    params = np.zeros((B, H, 2), dtype=np.float32)
    lib().dgqo_quantize_value(_p(V), C.c_int32(B), C.c_int32(nk), C.c_int32(H), C.c_int32(d),
                              C.c_int32(bits), _p(vhat), _p(codes), _p(params))
    return dict(vhat=vhat, codes=codes, params=params)


def xattn(Q, K, V, key_bias, bits: int, want_ahat: bool = False, s_in=None):
    """s_in [B]: a given (static) scale instead of the call's own maximum."""
    A = attn_probs(Q, K, key_bias)
    r = xattn_logq(A, V, bits, want_ahat, s_in=s_in)
    r["A"] = A
    return r


def xattn_intv(Q, K, V, key_bias):
    """The attention product of Section 3.3 on the INTEGER codes of V^, by shifts and adds
    (Section 3.1: the log quantizer "allows bit-shifting operations").  V^ = s_v q_v + z_v
    with 8-bit q_v (quantize_value); 4-bit probability codes A^q, so a quantized weight is
    s_b 2^-15 (1 << (15 - A^q)):
        acc[b,i,h,:] = sum_{j>=1} q_v[b,j,h,:] << (15 - A^q[b,h,i,j])        (integer)
        zsum[b,i,h]  = sum_{j>=1} 1 << (15 - A^q[b,h,i,j])                    (integer)
        out = A[..,0] * vhat[b,0,h,:] + s_b 2^-15 (s_v acc + z_v zsum)        (double, one rounding)
    Returns dict(out fp32 [B,N,H,d], acc int64 [B,N,H,d], zsum int64 [B,N,H], codes, s, margin)."""
    qv = quantize_value(V, 8)
    r = xattn(Q, K, qv["vhat"], key_bias, 4)
    codes = r["codes"].astype(np.int64)                       # [B,H,N,nk-1]
    shift = 15 - np.transpose(codes, (0, 2, 1, 3))            # [B,N,H,nk-1]
    vq = qv["codes"].astype(np.int64)[:, 1:]                  # [B,nk-1,H,d]
    B, N, H, _ = shift.shape
    d = vq.shape[-1]
    acc = np.zeros((B, N, H, d), np.int64)
    for j in range(shift.shape[-1]):                          # key by key: a shift and an add
        acc += vq[:, j][:, None, :, :] << shift[..., j][..., None]
    zsum = (np.int64(1) << shift).sum(-1)
    s_v = qv["params"][..., 0].astype(np.float64)[:, None, :, None]
    z_v = qv["params"][..., 1].astype(np.float64)[:, None, :, None]
    a0 = np.transpose(r["A"][..., 0], (0, 2, 1)).astype(np.float64)[..., None]   # [B,N,H,1]
    v0 = qv["vhat"][:, 0].astype(np.float64)[:, None]                              # [B,1,H,d]
    s_b = r["s"].astype(np.float64)[:, None, None, None]
    out = a0 * v0 + s_b * 2.0 ** -15 * (s_v * acc + z_v * zsum[..., None])
    return dict(out=out.astype(np.float32), acc=acc, zsum=zsum, codes=r["codes"], s=r["s"],
                margin=r["margin"], vq=qv)
