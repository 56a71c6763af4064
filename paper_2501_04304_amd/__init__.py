"""Python binding of libdgq.so (the MI355X DGQ quantized-inference library).

Argument marshalling only: every function below forwards torch device
tensors' pointers and sizes to the C entry point of the same name
(include/dgq.h).  There is no CPU fallback: if the HIP library is missing or a
call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libdgq.so")

DGQ_K_GRANULE = 64

_lib = None


class DgqError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("dgq error %d: %s" % (code, msg))
        self.code = code


class GroupsInfo(C.Structure):
    _fields_ = [("channels", C.c_int32), ("act_bits", C.c_int32), ("group_size", C.c_int32),
                ("n_pixel_classes", C.c_int32), ("n_groups", C.c_int32), ("k_padded", C.c_int32),
                ("n_outlier_channels", C.c_int32), ("n_regular_groups", C.c_int32),
                ("dstar", C.c_int32), ("code_offset", C.c_int32), ("n_class1_rows", C.c_int32),
                ("tau_pix", C.c_float), ("d_channel", C.c_double), ("d_pixel", C.c_double),
                ("grouping", C.c_int32), ("reserved", C.c_int32)]


DIM_AUTO, DIM_CHANNEL, DIM_PIXEL = -1, 0, 1
GROUPING_GRID, GROUPING_CHANNEL, GROUPING_PIXEL = 0, 1, 2


def lib():
    """Load libdgq.so; fail loudly when it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                "libdgq.so is not built: run `python -m paper_2501_04304_amd.build` "
                "(or __graft_entry__.build()) first")
        L = C.CDLL(LIB_PATH)
        vp, i32, i64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
        L.dgq_calibrate_groups.argtypes = [vp, i64, i32, i32, i32, i32, vp, C.POINTER(vp)]
        L.dgq_calibrate_kmeans.argtypes = [vp, i64, i32, i32, i32, i32, vp, C.POINTER(vp)]
        L.dgq_groups_thresholds.argtypes = [vp, vp]
        L.dgq_groups_info.argtypes = [vp, C.POINTER(GroupsInfo)]
        L.dgq_groups_tables.argtypes = [vp, vp, vp, vp, vp, vp]
        L.dgq_groups_free.argtypes = [vp]
        L.dgq_groups_free.restype = None
        L.dgq_pack_weight.argtypes = [vp, vp, vp, i32, i32, vp, C.POINTER(vp)]
        L.dgq_weight_tables.argtypes = [vp, vp, vp]
        L.dgq_weight_free.argtypes = [vp]
        L.dgq_weight_free.restype = None
        L.dgq_weight_pack_nibbles.argtypes = [vp, vp]
        L.dgq_weight_device_bytes.argtypes = [vp]
        L.dgq_weight_device_bytes.restype = sz
        L.dgq_quantize_act.argtypes = [vp, vp, i64, vp, vp, vp]
        L.dgq_linear.argtypes = [vp, vp, vp, vp, i64, vp, vp, vp, sz, vp]
        L.dgq_linear_geglu.argtypes = [vp, vp, vp, vp, i64, vp, vp]
        L.dgq_pack_weight_gated_for.argtypes = [vp, vp, vp, vp, i32, i32, vp, C.POINTER(vp)]
        L.dgq_linear_geglu_requant.argtypes = [vp, vp, vp, vp, i64, vp, vp, vp]
        L.dgq_groups_for_conv3x3.argtypes = [vp, C.POINTER(vp)]
        L.dgq_conv3x3_codes.argtypes = [vp, vp, i32, i32, i32, vp, vp]
        L.dgq_conv3x3_codes3_bytes.argtypes = [vp, i32, i32, i32]
        L.dgq_conv3x3_codes3_bytes.restype = sz
        L.dgq_quantize_act_conv3x3.argtypes = [vp, vp, vp, i32, i32, i32, vp, vp, vp]
        L.dgq_linear_conv3x3.argtypes = [vp, vp, vp, vp, i32, i32, i32, vp, vp]
        L.dgq_codes_bytes.argtypes = [vp, i64]
        L.dgq_codes_bytes.restype = sz
        L.dgq_linear_workspace_bytes.argtypes = [vp, vp, i64]
        L.dgq_linear_workspace_bytes.restype = sz
        L.dgq_xattn_logq.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, vp, vp, vp,
                                     vp, sz, vp]
        L.dgq_xattn_workspace_bytes.argtypes = [i32, i32, i32, i32, i32]
        L.dgq_xattn_logq_noalloc.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, vp, vp,
                                             vp, vp]
        L.dgq_quantize_value.argtypes = [vp, i32, i32, i32, i32, i32, vp, vp, vp, vp]
        L.dgq_xattn_logq_static.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, vp, vp, vp,
                                            vp, vp]
        L.dgq_xattn_workspace_bytes.restype = sz
        L.dgq_xattn_logq_intv.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp]
        L.dgq_selfattn_workspace_bytes.argtypes = [i32, i32, i32, i32]
        L.dgq_selfattn_workspace_bytes.restype = sz
        L.dgq_selfattn_logq.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, sz, vp]
        L.dgq_last_error.restype = C.c_char_p
        L.dgq_version.restype = C.c_int
        _lib = L
    return _lib


def _check(rc):
    if rc != 0:
        raise DgqError(rc, lib().dgq_last_error().decode())


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(stream=None):
    import torch
    s = stream if stream is not None else torch.cuda.current_stream()
    return C.c_void_p(s.cuda_stream)


def _dev(t, dtype, name):
    import torch
    if not isinstance(t, torch.Tensor) or not t.is_cuda or t.dtype != dtype or not t.is_contiguous():
        raise TypeError("%s must be a contiguous CUDA tensor of dtype %s" % (name, dtype))
    return t


@dataclass
class Groups:
    """Owner of a dgq_groups_t handle."""
    handle: int
    info: GroupsInfo

    def tables(self):
        import numpy as np
        ng, kp = self.info.n_groups, self.info.k_padded
        perm = np.empty(kp, np.int32)
        goff = np.empty(ng + 1, np.int32)
        glen = np.empty(ng, np.int32)
        p = max(self.info.n_pixel_classes, 2)
        s = np.empty((p, ng), np.float32)
        z = np.empty((p, ng), np.float32)
        _check(lib().dgq_groups_tables(self.handle, perm.ctypes.data, goff.ctypes.data,
                                       glen.ctypes.data, s.ctypes.data, z.ctypes.data))
        taus = np.empty(max(self.info.n_pixel_classes - 1, 1), np.float32)
        taus[:] = np.inf
        _check(lib().dgq_groups_thresholds(self.handle, taus.ctypes.data))
        return dict(perm=perm, goff=goff, glen=glen, s=s, z=z,
                    taus=taus[:max(self.info.n_pixel_classes - 1, 0)])

    def free(self):
        if self.handle:
            lib().dgq_groups_free(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


@dataclass
class Weight:
    """Owner of a dgq_weight_t handle."""
    handle: int
    groups: Groups
    out_channels: int
    w_bits: int

    def tables(self):
        import numpy as np
        wq = np.empty((self.out_channels, self.groups.info.channels), np.int8)
        sw = np.empty(self.out_channels, np.float32)
        _check(lib().dgq_weight_tables(self.handle, wq.ctypes.data, sw.ctypes.data))
        return dict(wq=wq, sw=sw)

    def pack_nibbles(self, stream=None):
        """Two 4-bit weights per byte (dgq_weight_pack_nibbles); dgq_linear then needs a workspace."""
        _check(lib().dgq_weight_pack_nibbles(self.handle, _stream(stream)))
        return self

    def device_bytes(self) -> int:
        return int(lib().dgq_weight_device_bytes(self.handle))

    def free(self):
        if self.handle:
            lib().dgq_weight_free(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def dgq_calibrate_groups(x_cal, act_bits: int, group_size: int, n_pixel_classes: int = 2,
                         stream=None) -> Groups:
    import torch
    _dev(x_cal, torch.float32, "x_cal")
    rows, ch = x_cal.shape
    h = C.c_void_p()
    _check(lib().dgq_calibrate_groups(_ptr(x_cal), rows, ch, act_bits, group_size,
                                      n_pixel_classes, _stream(stream), C.byref(h)))
    info = GroupsInfo()
    _check(lib().dgq_groups_info(h, C.byref(info)))
    return Groups(handle=h.value, info=info)


def dgq_calibrate_kmeans(x_cal, act_bits: int, n_clusters: int, dimension: int = DIM_AUTO,
                         stream=None) -> Groups:
    import torch
    _dev(x_cal, torch.float32, "x_cal")
    rows, ch = x_cal.shape
    h = C.c_void_p()
    _check(lib().dgq_calibrate_kmeans(_ptr(x_cal), rows, ch, act_bits, n_clusters, dimension,
                                      _stream(stream), C.byref(h)))
    info = GroupsInfo()
    _check(lib().dgq_groups_info(h, C.byref(info)))
    return Groups(handle=h.value, info=info)


def dgq_groups_for_conv3x3(groups: Groups) -> Groups:
    """The group tables of the 3 x 3 convolution over a map grouped by `groups` (one pixel
    class): nine replicated taps, 9 C channels."""
    h = C.c_void_p()
    _check(lib().dgq_groups_for_conv3x3(groups.handle, C.byref(h)))
    info = GroupsInfo()
    _check(lib().dgq_groups_info(h, C.byref(info)))
    return Groups(handle=h.value, info=info)


def dgq_conv3x3_codes(groups9: Groups, codes, B: int, H: int, W: int, codes9=None, stream=None):
    """codes of the [B*H*W, C] map (dgq_quantize_act) -> the unfolded codes of its 3 x 3
    convolution, int8 in the layout of codes_shape(groups9, B*H*W)."""
    import torch
    _dev(codes, torch.int8, "codes")
    rows = B * H * W
    shape = codes_shape(groups9, rows)
    if codes.numel() * 9 != shape[0] * shape[1] * shape[2]:
        raise ValueError("codes do not belong to a [B*H*W, C] map of this layer")
    if codes9 is None:
        codes9 = torch.empty(shape, dtype=torch.int8, device=codes.device)
    _dev(codes9, torch.int8, "codes9")
    if tuple(codes9.shape) != shape:
        raise ValueError("codes9 has the wrong shape")
    _check(lib().dgq_conv3x3_codes(groups9.handle, _ptr(codes), B, H, W, _ptr(codes9), _stream(stream)))
    return codes9


def dgq_quantize_act_conv3x3(groups: Groups, groups9: Groups, x, B: int, H: int, W: int, codes3=None,
                             row_class=None, stream=None):
    """x fp32 [B*H*W, C] -> (codes3, row_class): the three shifted copies of the map's codes that
    dgq_linear_conv3x3 gathers its nine taps from."""
    import torch
    _dev(x, torch.float32, "x")
    rows = B * H * W
    if tuple(x.shape) != (rows, groups.info.channels):
        raise ValueError("x must be [B*H*W, C]")
    nbytes = int(lib().dgq_conv3x3_codes3_bytes(groups9.handle, B, H, W))
    if codes3 is None:
        codes3 = torch.empty(nbytes, dtype=torch.int8, device=x.device)
    if row_class is None:
        row_class = torch.empty(rows, dtype=torch.uint8, device=x.device)
    _dev(codes3, torch.int8, "codes3")
    _dev(row_class, torch.uint8, "row_class")
    if codes3.numel() != nbytes or row_class.numel() != rows:
        raise ValueError("codes3 / row_class have the wrong size")
    _check(lib().dgq_quantize_act_conv3x3(groups.handle, groups9.handle, _ptr(x), B, H, W, _ptr(codes3),
                                          _ptr(row_class), _stream(stream)))
    return codes3, row_class


def dgq_linear_conv3x3(groups9: Groups, weight: "Weight", codes3, row_class, B: int, H: int, W: int, y=None,
                       stream=None):
    """The 3 x 3 convolution with its taps gathered by the contraction's loads: y fp32 [B*H*W, O]."""
    import torch
    _dev(codes3, torch.int8, "codes3")
    _dev(row_class, torch.uint8, "row_class")
    rows = B * H * W
    if y is None:
        y = torch.empty((rows, weight.out_channels), dtype=torch.float32, device=codes3.device)
    _dev(y, torch.float32, "y")
    if tuple(y.shape) != (rows, weight.out_channels):
        raise ValueError("y has the wrong shape")
    _check(lib().dgq_linear_conv3x3(groups9.handle, weight.handle, _ptr(codes3), _ptr(row_class), B, H, W,
                                    _ptr(y), _stream(stream)))
    return y


def dgq_pack_weight(groups: Groups, w, bias, w_bits: int, stream=None) -> Weight:
    import torch
    _dev(w, torch.float32, "w")
    if bias is not None:
        _dev(bias, torch.float32, "bias")
    O, ch = w.shape
    if ch != groups.info.channels:
        raise ValueError("w has %d input channels, the groups have %d" % (ch, groups.info.channels))
    h = C.c_void_p()
    _check(lib().dgq_pack_weight(groups.handle, _ptr(w), _ptr(bias), O, w_bits, _stream(stream),
                                 C.byref(h)))
    return Weight(handle=h.value, groups=groups, out_channels=O, w_bits=w_bits)


def dgq_pack_weight_gated_for(groups: Groups, next_groups: Groups, w, bias, w_bits: int,
                              stream=None) -> Weight:
    """Weights [value rows | gate rows] of a gated layer whose output is the input of the
    layer `next_groups` describes; for dgq_linear_geglu_requant."""
    import torch
    _dev(w, torch.float32, "w")
    if bias is not None:
        _dev(bias, torch.float32, "bias")
    O, ch = w.shape
    if ch != groups.info.channels:
        raise ValueError("w has %d input channels, the groups have %d" % (ch, groups.info.channels))
    h = C.c_void_p()
    _check(lib().dgq_pack_weight_gated_for(groups.handle, next_groups.handle, _ptr(w), _ptr(bias), O,
                                           w_bits, _stream(stream), C.byref(h)))
    return Weight(handle=h.value, groups=groups, out_channels=O, w_bits=w_bits)


def codes_shape(groups: Groups, rows: int):
    """Shape of the block-tiled code buffer: [row blocks, chunks, 1024 bytes]."""
    n_chunks = groups.info.k_padded // DGQ_K_GRANULE
    nbytes = int(lib().dgq_codes_bytes(groups.handle, rows))
    return (nbytes // (n_chunks * 1024), n_chunks, 1024)


def dgq_quantize_act(groups: Groups, x, codes=None, row_class=None, stream=None):
    """Returns (codes int8 [row blocks, chunks, 1024] block-tiled, row_class uint8 [rows])."""
    import torch
    _dev(x, torch.float32, "x")
    rows, ch = x.shape
    if ch != groups.info.channels:
        raise ValueError("x has %d channels, the groups have %d" % (ch, groups.info.channels))
    if codes is None:
        codes = torch.empty(codes_shape(groups, rows), dtype=torch.int8, device=x.device)
    if row_class is None:
        row_class = torch.empty(rows, dtype=torch.uint8, device=x.device)
    _dev(codes, torch.int8, "codes")
    _dev(row_class, torch.uint8, "row_class")
    if tuple(codes.shape) != codes_shape(groups, rows) or row_class.numel() != rows:
        raise ValueError("codes / row_class have the wrong shape")
    _check(lib().dgq_quantize_act(groups.handle, _ptr(x), rows, _ptr(codes), _ptr(row_class),
                                  _stream(stream)))
    return codes, row_class


def dgq_linear_workspace_bytes(groups: Groups, weight: Weight, rows: int) -> int:
    return int(lib().dgq_linear_workspace_bytes(groups.handle, weight.handle, rows))


def dgq_linear(groups: Groups, weight: Weight, codes, row_class, y=None, acc_dump=None,
               stream=None, workspace=None):
    """Returns y fp32 [rows, O]; acc_dump (optional) int32 [rows, O, NG] is filled in place.
    workspace: uint8 device tensor of dgq_linear_workspace_bytes() bytes (nibble-packed weights)."""
    import torch
    _dev(codes, torch.int8, "codes")
    _dev(row_class, torch.uint8, "row_class")
    rows = row_class.numel()
    if tuple(codes.shape) != codes_shape(groups, rows):
        raise ValueError("codes / row_class have the wrong shape")
    O = weight.out_channels
    if y is None:
        y = torch.empty((rows, O), dtype=torch.float32, device=codes.device)
    _dev(y, torch.float32, "y")
    if tuple(y.shape) != (rows, O):
        raise ValueError("y has the wrong shape")
    if acc_dump is not None:
        _dev(acc_dump, torch.int32, "acc_dump")
        if tuple(acc_dump.shape) != (rows, O, groups.info.n_groups):
            raise ValueError("acc_dump has the wrong shape")
    ws_ptr, ws_bytes = None, 0
    if workspace is not None:
        _dev(workspace, torch.uint8, "workspace")
        ws_ptr, ws_bytes = _ptr(workspace), workspace.numel()
    _check(lib().dgq_linear(groups.handle, weight.handle, _ptr(codes), _ptr(row_class), rows,
                            _ptr(y), _ptr(acc_dump), ws_ptr, ws_bytes, _stream(stream)))
    return y


def dgq_linear_geglu(groups: Groups, weight: Weight, codes, row_class, y=None, stream=None):
    """Returns fp32 [rows, O / 2]: first half of the layer's outputs times GELU(second half)."""
    import torch
    _dev(codes, torch.int8, "codes")
    _dev(row_class, torch.uint8, "row_class")
    rows = row_class.numel()
    if tuple(codes.shape) != codes_shape(groups, rows):
        raise ValueError("codes / row_class have the wrong shape")
    oh = weight.out_channels // 2
    if y is None:
        y = torch.empty((rows, oh), dtype=torch.float32, device=codes.device)
    _dev(y, torch.float32, "y")
    if tuple(y.shape) != (rows, oh):
        raise ValueError("y has the wrong shape")
    _check(lib().dgq_linear_geglu(groups.handle, weight.handle, _ptr(codes), _ptr(row_class),
                                  rows, _ptr(y), _stream(stream)))
    return y


def dgq_linear_geglu_requant(groups: Groups, weight: Weight, codes, row_class, next_groups: Groups,
                             codes_next=None, row_class_next=None, stream=None):
    """Returns (codes_next, row_class_next): the following layer's codes of
    value * GELU(gate), in the layout of dgq_quantize_act(next_groups, .)."""
    import torch
    _dev(codes, torch.int8, "codes")
    _dev(row_class, torch.uint8, "row_class")
    rows = row_class.numel()
    if tuple(codes.shape) != codes_shape(groups, rows):
        raise ValueError("codes / row_class have the wrong shape")
    shape = codes_shape(next_groups, rows)
    if codes_next is None:
        codes_next = torch.empty(shape, dtype=torch.int8, device=codes.device)
    if row_class_next is None:
        row_class_next = torch.empty(rows, dtype=torch.uint8, device=codes.device)
    _dev(codes_next, torch.int8, "codes_next")
    _dev(row_class_next, torch.uint8, "row_class_next")
    if tuple(codes_next.shape) != shape or row_class_next.numel() != rows:
        raise ValueError("codes_next / row_class_next have the wrong shape")
    _check(lib().dgq_linear_geglu_requant(groups.handle, weight.handle, _ptr(codes), _ptr(row_class),
                                          rows, _ptr(codes_next), _ptr(row_class_next),
                                          _stream(stream)))
    return codes_next, row_class_next


def dgq_xattn_workspace_bytes(B, N, H, d, nk) -> int:
    return int(lib().dgq_xattn_workspace_bytes(B, N, H, d, nk))


def dgq_xattn_logq(q, k, v, key_bias, attn_bits: int, out=None, scale_out=None, codes_dump=None,
                   workspace=None, stream=None):
    """q [B,N,H,d], k/v [B,nk,H,d] -> (out [B,N,H,d], scale [B])."""
    import torch
    _dev(q, torch.float32, "q")
    _dev(k, torch.float32, "k")
    _dev(v, torch.float32, "v")
    if key_bias is not None:
        _dev(key_bias, torch.float32, "key_bias")
    B, N, H, d = q.shape
    nk = k.shape[1]
    if tuple(k.shape) != (B, nk, H, d) or tuple(v.shape) != (B, nk, H, d):
        raise ValueError("k / v have the wrong shape")
    if key_bias is not None and key_bias.numel() != nk:
        raise ValueError("key_bias has the wrong shape")
    if out is None:
        out = torch.empty_like(q)
    if scale_out is None:
        scale_out = torch.empty(B, dtype=torch.float32, device=q.device)
    _dev(out, torch.float32, "out")
    _dev(scale_out, torch.float32, "scale_out")
    if codes_dump is not None:
        _dev(codes_dump, torch.uint8, "codes_dump")
        if tuple(codes_dump.shape) != (B, H, N, nk - 1):
            raise ValueError("codes_dump has the wrong shape")
    need = dgq_xattn_workspace_bytes(B, N, H, d, nk)
    if workspace is None and need:
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    wbytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib().dgq_xattn_logq(_ptr(q), _ptr(k), _ptr(v), _ptr(key_bias), B, N, H, d, nk,
                                attn_bits, _ptr(out), _ptr(scale_out), _ptr(codes_dump),
                                _ptr(workspace), wbytes, _stream(stream)))
    return out, scale_out


def dgq_xattn_logq_intv(q, k, v_codes, v_params, key_bias, attn_bits: int = 4, out=None, scale_out=None,
                        codes_dump=None, acc_dump=None, stream=None):
    """Attention product on the integer codes of V^ (u8 [B,nk,H,d]) and their (s, z) [B,H,2]."""
    import torch
    _dev(q, torch.float32, "q")
    _dev(k, torch.float32, "k")
    _dev(v_codes, torch.uint8, "v_codes")
    _dev(v_params, torch.float32, "v_params")
    B, N, H, d = q.shape
    nk = k.shape[1]
    if tuple(k.shape) != (B, nk, H, d) or tuple(v_codes.shape) != (B, nk, H, d):
        raise ValueError("k / v_codes have the wrong shape")
    if v_params.numel() != B * H * 2:
        raise ValueError("v_params must be [B, H, 2]")
    if out is None:
        out = torch.empty_like(q)
    if scale_out is None:
        scale_out = torch.empty(B, dtype=torch.float32, device=q.device)
    if acc_dump is not None:
        _dev(acc_dump, torch.int32, "acc_dump")
        if tuple(acc_dump.shape) != (B, N, H, d):
            raise ValueError("acc_dump has the wrong shape")
    if codes_dump is not None:
        _dev(codes_dump, torch.uint8, "codes_dump")
        if tuple(codes_dump.shape) != (B, H, N, nk - 1):
            raise ValueError("codes_dump has the wrong shape")
    _check(lib().dgq_xattn_logq_intv(_ptr(q), _ptr(k), _ptr(v_codes), _ptr(v_params), _ptr(key_bias), B, N,
                                     H, d, nk, attn_bits, _ptr(out), _ptr(scale_out), _ptr(codes_dump),
                                     _ptr(acc_dump), _stream(stream)))
    return out, scale_out


XATTN_NOALLOC_MAX_ROWS = 1 << 20


def dgq_xattn_logq_noalloc(q, k, v, key_bias, attn_bits: int, out, scale_out, codes_dump=None,
                           stream=None):
    """dgq_xattn_logq without a workspace: the caller passes every buffer (out [B,N,H,d],
    scale_out [B]) and nothing is allocated, here or in the library."""
    import torch
    for t, name in ((q, "q"), (k, "k"), (v, "v"), (out, "out"), (scale_out, "scale_out")):
        _dev(t, torch.float32, name)
    if key_bias is not None:
        _dev(key_bias, torch.float32, "key_bias")
    B, N, H, d = q.shape
    nk = k.shape[1]
    if tuple(k.shape) != (B, nk, H, d) or tuple(v.shape) != (B, nk, H, d):
        raise ValueError("k / v have the wrong shape")
    if tuple(out.shape) != (B, N, H, d) or scale_out.numel() != B:
        raise ValueError("out / scale_out have the wrong shape")
    if key_bias is not None and key_bias.numel() != nk:
        raise ValueError("key_bias has the wrong shape")
    if codes_dump is not None:
        _dev(codes_dump, torch.uint8, "codes_dump")
        if tuple(codes_dump.shape) != (B, H, N, nk - 1):
            raise ValueError("codes_dump has the wrong shape")
    _check(lib().dgq_xattn_logq_noalloc(_ptr(q), _ptr(k), _ptr(v), _ptr(key_bias), B, N, H, d, nk,
                                        attn_bits, _ptr(out), _ptr(scale_out), _ptr(codes_dump),
                                        _stream(stream)))
    return out, scale_out


def dgq_selfattn_workspace_bytes(B, N, H, d) -> int:
    return int(lib().dgq_selfattn_workspace_bytes(B, N, H, d))


def dgq_selfattn_logq(q, k, v, attn_bits: int, scale_in, out=None, scale_out=None, codes_dump=None,
                      workspace=None, stream=None):
    """q, k, v fp32 [B,N,H,d], scale_in fp32 [B] -> out fp32 [B,N,H,d].  scale_out [B] and
    codes_dump u8 [B,H,N,N] are filled if given."""
    import torch
    for t, name in ((q, "q"), (k, "k"), (v, "v"), (scale_in, "scale_in")):
        _dev(t, torch.float32, name)
    B, N, H, d = q.shape
    if tuple(k.shape) != (B, N, H, d) or tuple(v.shape) != (B, N, H, d) or scale_in.numel() != B:
        raise ValueError("q, k, v must share one shape [B,N,H,d] and scale_in have B entries")
    if out is None:
        out = torch.empty_like(q)
    _dev(out, torch.float32, "out")
    if scale_out is not None:
        _dev(scale_out, torch.float32, "scale_out")
    if codes_dump is not None:
        _dev(codes_dump, torch.uint8, "codes_dump")
        if tuple(codes_dump.shape) != (B, H, N, N):
            raise ValueError("codes_dump must be [B,H,N,N]")
    need = dgq_selfattn_workspace_bytes(B, N, H, d)
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=q.device)
    _check(lib().dgq_selfattn_logq(_ptr(q), _ptr(k), _ptr(v), B, N, H, d, attn_bits, _ptr(scale_in),
                                   _ptr(out), _ptr(scale_out), _ptr(codes_dump), _ptr(workspace),
                                   workspace.numel(), _stream(stream)))
    return out


def dgq_quantize_value(v, v_bits: int = 8, v_hat=None, want_codes: bool = False,
                       want_params: bool = False, stream=None):
    """v [B,nk,H,d] fp32 -> v_hat (and, on request, the codes and the (s, z) pairs)."""
    import torch
    _dev(v, torch.float32, "v")
    B, nk, H, d = v.shape
    if v_hat is None:
        v_hat = torch.empty_like(v)
    codes = torch.empty(v.shape, dtype=torch.uint8, device=v.device) if want_codes else None
    params = torch.empty((B, H, 2), dtype=torch.float32, device=v.device) if want_params else None
    _check(lib().dgq_quantize_value(_ptr(v), B, nk, H, d, v_bits, _ptr(v_hat),
                                    _ptr(codes) if codes is not None else None,
                                    _ptr(params) if params is not None else None, _stream(stream)))
    return v_hat, codes, params


def dgq_xattn_logq_static(q, k, v, key_bias, attn_bits: int, scale_in, out=None, scale_out=None,
                          codes_dump=None, stream=None):
    """Attention with a given prompt scale (one pass).  Returns (out, scale_out or None)."""
    import torch
    _dev(q, torch.float32, "q")
    _dev(k, torch.float32, "k")
    _dev(v, torch.float32, "v")
    _dev(scale_in, torch.float32, "scale_in")
    B, N, H, d = q.shape
    nk = k.shape[1]
    if out is None:
        out = torch.empty_like(q)
    _check(lib().dgq_xattn_logq_static(_ptr(q), _ptr(k), _ptr(v),
                                       _ptr(key_bias) if key_bias is not None else None, B, N, H, d,
                                       nk, attn_bits, _ptr(scale_in), _ptr(out),
                                       _ptr(scale_out) if scale_out is not None else None,
                                       _ptr(codes_dump) if codes_dump is not None else None,
                                       _stream(stream)))
    return out, scale_out
