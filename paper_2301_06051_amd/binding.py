"""ctypes binding of libdsvt.so: argument marshalling only.

Every step of the path runs inside the HIP library; PyTorch supplies device memory and the
stream.  There is no CPU fallback: a missing library raises.
"""
import ctypes as C
import os

import numpy as np
import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libdsvt.so")

DSVT_OK, DSVT_EINVAL, DSVT_ENOSPC, DSVT_EHIP, DSVT_EUNSUPPORTED = 0, -1, -2, -3, -4
DSVT_F32, DSVT_BF16 = 0, 1
ST_COORD_RANGE, ST_COORD_REPEAT, ST_SET_OVERFLOW, ST_WS_STATE, ST_VOXEL_OVERFLOW, ST_TILE_OVERFLOW = 1, 2, 4, 8, 16, 32
_ERR = {-1: "DSVT_EINVAL", -2: "DSVT_ENOSPC", -3: "DSVT_EHIP", -4: "DSVT_EUNSUPPORTED"}
_DT = {"f32": (DSVT_F32, torch.float32), "bf16": (DSVT_BF16, torch.bfloat16)}

I32x3 = C.c_int32 * 3
F32x3 = C.c_float * 3


class PartCfg(C.Structure):
    _fields_ = [("grid", I32x3), ("win", I32x3), ("shift", I32x3), ("tau", C.c_int32), ("batch", C.c_int32),
                ("axis", C.c_int32)]


class TileList(C.Structure):
    _fields_ = [("max_tiles", C.c_int32), ("tile_first", C.c_void_p), ("n_tiles", C.c_void_p),
                ("tile_order", C.c_void_p), ("tile_desc", C.c_void_p)]


class XyJob(C.Structure):
    _fields_ = [("cfg", PartCfg), ("set_inds_x", C.c_void_p), ("set_inds_y", C.c_void_p), ("voxel_slot_x", C.c_void_p),
                ("voxel_slot_y", C.c_void_p), ("n_sets", C.c_void_p), ("set_win", C.c_void_p), ("max_sets", C.c_int32),
                ("tiles", C.POINTER(TileList)), ("tile_desc_y", C.c_void_p), ("ws", C.c_void_p), ("ws_bytes", C.c_size_t),
                ("status", C.c_void_p)]


class Maps(C.Structure):
    _fields_ = [("n_voxels", C.c_int32), ("max_sets", C.c_int32), ("tau", C.c_int32), ("set_inds", C.c_void_p),
                ("voxel_slot", C.c_void_p), ("n_sets", C.c_void_p), ("tiles", TileList)]


class LayerW(C.Structure):
    _fields_ = [("C", C.c_int32), ("heads", C.c_int32), ("hidden", C.c_int32), ("dtype", C.c_int32),
                ("w_qkv", C.c_void_p), ("w_o", C.c_void_p), ("w_1", C.c_void_p), ("w_2", C.c_void_p),
                ("b_qkv", C.c_void_p), ("b_o", C.c_void_p), ("b_1", C.c_void_p), ("b_2", C.c_void_p),
                ("ln1_g", C.c_void_p), ("ln1_b", C.c_void_p), ("ln2_g", C.c_void_p), ("ln2_b", C.c_void_p),
                ("ln_eps", C.c_float), ("rel_bias", C.c_void_p), ("win", I32x3), ("dup_mode", C.c_int32),
                ("packed", C.c_void_p)]


class VfeCfg(C.Structure):
    _fields_ = [("grid", I32x3), ("batch", C.c_int32), ("range_min", F32x3), ("voxel_size", F32x3), ("f_in", C.c_int32),
                ("C", C.c_int32), ("dtype", C.c_int32), ("w", C.c_void_p), ("b", C.c_void_p), ("relu", C.c_int32)]


class PoolCfg(C.Structure):
    _fields_ = [("grid", I32x3), ("pool", I32x3), ("batch", C.c_int32), ("C", C.c_int32), ("heads", C.c_int32),
                ("dtype", C.c_int32), ("w_q", C.c_void_p), ("w_k", C.c_void_p), ("w_v", C.c_void_p),
                ("w_o", C.c_void_p), ("b_q", C.c_void_p), ("b_k", C.c_void_p), ("b_v", C.c_void_p),
                ("b_o", C.c_void_p), ("ln_g", C.c_void_p), ("ln_b", C.c_void_p), ("ln_eps", C.c_float),
                ("mask_empty", C.c_int32), ("packed", C.c_void_p)]


_lib = None


def lib():
    """The loaded C-ABI library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                               "(there is no fallback path)")
        L = C.CDLL(LIB_PATH)
        vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
        L.dsvt_partition_bound.argtypes = [C.POINTER(PartCfg), i32, C.POINTER(i32), C.POINTER(i32), C.POINTER(sz)]
        L.dsvt_partition.argtypes = [C.POINTER(PartCfg), vp, i32, vp, vp, vp, i32, vp, C.POINTER(TileList), vp, sz, vp, vp]
        L.dsvt_partition_ws_init.argtypes = [C.POINTER(PartCfg), i32, vp, sz, vp]
        L.dsvt_partition_xy.argtypes = [C.POINTER(PartCfg), vp, i32, vp, vp, vp, vp, vp, i32, vp, C.POINTER(TileList), vp,
                                        vp, sz, vp, vp]
        L.dsvt_partition_xy_multi.argtypes = [C.POINTER(XyJob), i32, vp, i32, vp]
        L.dsvt_layer_packed_size.argtypes = [C.POINTER(LayerW), C.POINTER(sz)]
        L.dsvt_layer_pack.argtypes = [C.POINTER(LayerW), vp, sz, vp]
        L.dsvt_block_workspace_size.argtypes = [C.POINTER(LayerW), i32, C.POINTER(sz)]
        L.dsvt_set_attention_workspace_size.argtypes = [C.POINTER(LayerW), i32, C.POINTER(sz)]
        L.dsvt_set_attention.argtypes = [C.POINTER(LayerW), C.POINTER(Maps), vp, vp, vp, vp, sz, vp]
        L.dsvt_block.argtypes = [C.POINTER(LayerW), C.POINTER(Maps), vp, vp, vp, vp, sz, vp]
        L.dsvt_pool_packed_size.argtypes = [C.POINTER(PoolCfg), C.POINTER(sz)]
        L.dsvt_pool_pack.argtypes = [C.POINTER(PoolCfg), vp, sz, vp]
        L.dsvt_attn_pool_workspace_size.argtypes = [C.POINTER(PoolCfg), i32, C.POINTER(sz)]
        L.dsvt_attn_pool.argtypes = [C.POINTER(PoolCfg), vp, vp, i32, vp, vp, vp, vp, sz, vp, vp]
        L.dsvt_attn_pool_static.argtypes = [C.POINTER(PoolCfg), vp, vp, i32, vp, vp, vp, vp, vp]
        L.dsvt_bev_scatter.argtypes = [vp, vp, i32, i32, i32, i32, C.POINTER(I32x3), vp, vp, vp]
        L.dsvt_vfe_workspace_size.argtypes = [C.POINTER(VfeCfg), i32, i32, C.POINTER(sz)]
        L.dsvt_vfe.argtypes = [C.POINTER(VfeCfg), vp, vp, i32, vp, vp, vp, i32, vp, sz, vp, vp]
        L.dsvt_prof_enable.argtypes = [i32]
        L.dsvt_prof_collect.argtypes = [C.POINTER(C.c_float), C.POINTER(i32), i32]
        L.dsvt_prof_kernel_count.restype = i32
        L.dsvt_prof_kernel_name.argtypes = [i32]
        L.dsvt_prof_kernel_name.restype = C.c_char_p
        _lib = L
    return _lib


class DsvtError(RuntimeError):
    def __init__(self, where, rc):
        super().__init__(f"{where} returned {_ERR.get(rc, rc)}")
        self.rc = rc


def _check(where, rc):
    if rc != DSVT_OK:
        raise DsvtError(where, rc)


def _stream(stream):
    return C.c_void_p(torch.cuda.current_stream().cuda_stream if stream is None else stream)


def _ptr(t):
    return C.c_void_p(0 if t is None else t.data_ptr())


def _dev(a, dtype):
    return torch.as_tensor(np.ascontiguousarray(a)).to(device="cuda", dtype=dtype).contiguous()


def part_cfg(grid, win, shift, tau, batch, axis):
    return PartCfg(I32x3(*grid), I32x3(*win), I32x3(*shift), tau, batch, axis)


def dsvt_partition_bound(cfg, n_voxels):
    ms, mt, ws = C.c_int32(0), C.c_int32(0), C.c_size_t(0)
    _check("dsvt_partition_bound",
           lib().dsvt_partition_bound(C.byref(cfg), n_voxels, C.byref(ms), C.byref(mt), C.byref(ws)))
    return ms.value, mt.value, ws.value


class SetMaps:
    """Device buffers of one (window configuration, axis) and the struct the kernels read."""

    def __init__(self, cfg, n_voxels, max_sets=None, tiles=True, common=None, max_tiles=None):
        """common: the SetMaps of the other axis of the same dsvt_partition_xy call, whose n_sets, set_win,
        status, scratch and tile boundaries this one shares.  max_tiles: a work list shorter than the bound."""
        bound, tile_bound, ws_bytes = dsvt_partition_bound(cfg, n_voxels)
        self.cfg, self.n_voxels, self.tau = cfg, n_voxels, cfg.tau
        self.max_sets = bound if max_sets is None else max_sets
        i32 = dict(dtype=torch.int32, device="cuda")
        self.set_inds = torch.full((self.max_sets, cfg.tau), -1, **i32)
        self.voxel_slot = torch.full((n_voxels,), -1, **i32)
        if common is None:
            self.set_win = torch.full((self.max_sets,), -1, **i32)
            self.n_sets = torch.zeros((1,), **i32)
            self.status = torch.zeros((1,), **i32)
            self.ws = torch.empty((ws_bytes,), dtype=torch.uint8, device="cuda")
            _check("dsvt_partition_ws_init",
                   lib().dsvt_partition_ws_init(C.byref(cfg), n_voxels, _ptr(self.ws), ws_bytes, _stream(None)))
            torch.cuda.current_stream().synchronize()     # the maps may first be used on any stream
        else:
            assert common.max_sets == self.max_sets and common.n_voxels == n_voxels
            self.set_win, self.n_sets, self.status, self.ws = common.set_win, common.n_sets, common.status, common.ws
        self.max_tiles = tile_bound if (tiles and tile_bound > 0 and cfg.tau <= 96) else 0
        if self.max_tiles and max_tiles is not None:
            self.max_tiles = min(self.max_tiles, max_tiles)
        if self.max_tiles:
            if common is None:
                self.tile_first = torch.full((self.max_tiles + 1,), -1, **i32)
                self.n_tiles = torch.zeros((1,), **i32)
                self.tile_order = torch.full((self.max_tiles,), -1, **i32)
            else:
                self.tile_first, self.n_tiles, self.tile_order = common.tile_first, common.n_tiles, common.tile_order
            self.tile_desc = torch.full((self.max_tiles, 256), -1, **i32)
            self.tile_list = TileList(self.max_tiles, self.tile_first.data_ptr(), self.n_tiles.data_ptr(),
                                      self.tile_order.data_ptr(), self.tile_desc.data_ptr())
        else:
            self.tile_first = self.n_tiles = self.tile_order = self.tile_desc = None
            self.tile_list = TileList(0, None, None, None, None)
        self.struct = Maps(n_voxels, self.max_sets, cfg.tau, self.set_inds.data_ptr(), self.voxel_slot.data_ptr(),
                           self.n_sets.data_ptr(), self.tile_list)


def dsvt_partition(cfg, coords, out=None, stream=None):
    """coords: int32 cuda tensor [N,4].  Returns the SetMaps it filled (allocated here unless given)."""
    assert coords.is_cuda and coords.dtype == torch.int32 and coords.is_contiguous() and coords.shape[1] == 4
    n = coords.shape[0]
    out = SetMaps(cfg, n) if out is None else out
    assert out.n_voxels == n
    rc = lib().dsvt_partition(C.byref(cfg), _ptr(coords), n, _ptr(out.set_inds), _ptr(out.voxel_slot),
                              _ptr(out.n_sets), out.max_sets, _ptr(out.set_win),
                              C.byref(out.tile_list) if out.max_tiles else None, _ptr(out.ws), out.ws.numel(),
                              _ptr(out.status),
                              _stream(stream))
    _check("dsvt_partition", rc)
    return out


class SetMapsXY:
    """The maps of both axes of one window configuration, filled by one dsvt_partition_xy call; indexes
    and iterates like the pair [X-axis maps, Y-axis maps]."""

    def __init__(self, cfg, n_voxels, max_sets=None, tiles=True, max_tiles=None):
        self.x = SetMaps(cfg, n_voxels, max_sets, tiles, max_tiles=max_tiles)
        self.y = SetMaps(cfg, n_voxels, max_sets, tiles, common=self.x, max_tiles=max_tiles)
        self.n_voxels = n_voxels

    def __getitem__(self, k):
        return (self.x, self.y)[k]

    def __iter__(self):
        return iter((self.x, self.y))

    def __len__(self):
        return 2


def dsvt_partition_xy(cfg, coords, out=None, stream=None):
    """Both rotated partitions of one window configuration.  Returns the SetMapsXY it filled."""
    assert coords.is_cuda and coords.dtype == torch.int32 and coords.is_contiguous() and coords.shape[1] == 4
    n = coords.shape[0]
    out = SetMapsXY(cfg, n) if out is None else out
    assert out.n_voxels == n
    x, y = out.x, out.y
    rc = lib().dsvt_partition_xy(C.byref(cfg), _ptr(coords), n, _ptr(x.set_inds), _ptr(y.set_inds), _ptr(x.voxel_slot),
                                 _ptr(y.voxel_slot), _ptr(x.n_sets), x.max_sets, _ptr(x.set_win),
                                 C.byref(x.tile_list) if x.max_tiles else None, _ptr(y.tile_desc) if x.max_tiles else None,
                                 _ptr(x.ws), x.ws.numel(), _ptr(x.status), _stream(stream))
    _check("dsvt_partition_xy", rc)
    return out


def dsvt_partition_xy_multi(cfgs, coords, outs, stream=None):
    """The partitions of several window configurations (cfgs[k] into the SetMapsXY outs[k]) in one pass."""
    assert coords.is_cuda and coords.dtype == torch.int32 and coords.is_contiguous() and coords.shape[1] == 4
    n = coords.shape[0]
    assert len(cfgs) == len(outs) and all(o.n_voxels == n for o in outs)
    jobs = (XyJob * len(cfgs))()
    for j, cfg, o in zip(jobs, cfgs, outs):
        x, y = o.x, o.y
        j.cfg = cfg
        j.set_inds_x, j.set_inds_y = x.set_inds.data_ptr(), y.set_inds.data_ptr()
        j.voxel_slot_x, j.voxel_slot_y = x.voxel_slot.data_ptr(), y.voxel_slot.data_ptr()
        j.n_sets, j.set_win, j.max_sets = x.n_sets.data_ptr(), x.set_win.data_ptr(), x.max_sets
        j.tiles = C.pointer(x.tile_list) if x.max_tiles else None
        j.tile_desc_y = y.tile_desc.data_ptr() if x.max_tiles else None
        j.ws, j.ws_bytes, j.status = x.ws.data_ptr(), x.ws.numel(), x.status.data_ptr()
    _check("dsvt_partition_xy_multi", lib().dsvt_partition_xy_multi(jobs, len(cfgs), _ptr(coords), n, _stream(stream)))
    return outs


class LayerWeights:
    """Device copy of one DSVT layer's parameters (from a synth-style dict of numpy arrays)."""

    def __init__(self, w, dup_mode=0):
        code, tdt = _DT[w["dtype"]]
        f32 = torch.float32
        self.t = {k: _dev(w[k], tdt) for k in ("w_qkv", "w_o", "w_1", "w_2")}
        self.t.update({k: _dev(w[k], f32) for k in ("b_qkv", "b_o", "b_1", "b_2", "ln1_g", "ln1_b", "ln2_g", "ln2_b")})
        self.t["rel_bias"] = None if w.get("rel_bias") is None else _dev(w["rel_bias"], f32)
        self.dtype, self.C = tdt, w["C"]
        p = lambda k: self.t[k].data_ptr() if self.t[k] is not None else None
        self.struct = LayerW(w["C"], w["heads"], w["hidden"], code, p("w_qkv"), p("w_o"), p("w_1"), p("w_2"),
                             p("b_qkv"), p("b_o"), p("b_1"), p("b_2"), p("ln1_g"), p("ln1_b"), p("ln2_g"), p("ln2_b"),
                             w["ln_eps"], p("rel_bias"), I32x3(*w["win"]), dup_mode, None)
        nbytes = C.c_size_t(0)
        _check("dsvt_layer_packed_size", lib().dsvt_layer_packed_size(C.byref(self.struct), C.byref(nbytes)))
        self.packed = torch.empty((nbytes.value,), dtype=torch.uint8, device="cuda")
        _check("dsvt_layer_pack", lib().dsvt_layer_pack(C.byref(self.struct), _ptr(self.packed), nbytes.value, _stream(None)))
        self.struct.packed = self.packed.data_ptr()


def dsvt_set_attention_workspace_size(layer, n_voxels):
    sz = C.c_size_t(0)
    _check("dsvt_set_attention_workspace_size",
           lib().dsvt_set_attention_workspace_size(C.byref(layer.struct), n_voxels, C.byref(sz)))
    return sz.value


def dsvt_block_workspace_size(layer, n_voxels):
    sz = C.c_size_t(0)
    _check("dsvt_block_workspace_size", lib().dsvt_block_workspace_size(C.byref(layer.struct), n_voxels, C.byref(sz)))
    return sz.value


def _ws(nbytes, ws):
    if ws is None:
        ws = torch.empty((max(nbytes, 1),), dtype=torch.uint8, device="cuda")
    return ws


def dsvt_set_attention(layer, maps, coords, x, y=None, ws=None, stream=None):
    assert x.is_cuda and x.dtype == layer.dtype and x.is_contiguous() and x.shape == (maps.n_voxels, layer.C)
    y = torch.empty_like(x) if y is None else y
    ws = _ws(dsvt_block_workspace_size(layer, maps.n_voxels), ws)
    rc = lib().dsvt_set_attention(C.byref(layer.struct), C.byref(maps.struct), _ptr(coords), _ptr(x), _ptr(y),
                                  _ptr(ws), ws.numel(), _stream(stream))
    _check("dsvt_set_attention", rc)
    return y


def dsvt_block(layers, maps, coords, x_in, x_out=None, ws=None, stream=None):
    """layers: (X-axis LayerWeights, Y-axis LayerWeights); maps: (X-axis SetMaps, Y-axis SetMaps)."""
    assert x_in.is_cuda and x_in.dtype == layers[0].dtype and x_in.is_contiguous()
    x_out = torch.empty_like(x_in) if x_out is None else x_out
    ws = _ws(dsvt_block_workspace_size(layers[0], maps[0].n_voxels), ws)
    lw = (LayerW * 2)(layers[0].struct, layers[1].struct)
    mp = (Maps * 2)(maps[0].struct, maps[1].struct)
    rc = lib().dsvt_block(lw, mp, _ptr(coords), _ptr(x_in), _ptr(x_out), _ptr(ws), ws.numel(), _stream(stream))
    _check("dsvt_block", rc)
    return x_out


class PoolWeights:
    def __init__(self, w, grid, pool, batch, mask_empty=1):
        code, tdt = _DT[w["dtype"]]
        self.t = {k: _dev(w[k], tdt) for k in ("w_q", "w_k", "w_v", "w_o")}
        self.t.update({k: _dev(w[k], torch.float32) for k in ("b_q", "b_k", "b_v", "b_o", "ln_g", "ln_b")})
        self.dtype, self.C = tdt, w["C"]
        p = lambda k: self.t[k].data_ptr()
        self.struct = PoolCfg(I32x3(*grid), I32x3(*pool), batch, w["C"], w["heads"], code, p("w_q"), p("w_k"),
                              p("w_v"), p("w_o"), p("b_q"), p("b_k"), p("b_v"), p("b_o"), p("ln_g"), p("ln_b"),
                              w["ln_eps"], mask_empty, None)
        nbytes = C.c_size_t(0)
        _check("dsvt_pool_packed_size", lib().dsvt_pool_packed_size(C.byref(self.struct), C.byref(nbytes)))
        self.packed = torch.empty((nbytes.value,), dtype=torch.uint8, device="cuda")
        _check("dsvt_pool_pack", lib().dsvt_pool_pack(C.byref(self.struct), _ptr(self.packed), nbytes.value, _stream(None)))
        self.struct.packed = self.packed.data_ptr()


def dsvt_attn_pool_workspace_size(pool, n_voxels):
    sz = C.c_size_t(0)
    _check("dsvt_attn_pool_workspace_size",
           lib().dsvt_attn_pool_workspace_size(C.byref(pool.struct), n_voxels, C.byref(sz)))
    return sz.value


def dsvt_attn_pool(pool, coords, x, out=None, ws=None, stream=None):
    """Returns (out_coords [N,4], out [N,C], n_out device scalar, status); the first n_out rows are valid."""
    n = coords.shape[0]
    assert x.is_cuda and x.dtype == pool.dtype and x.is_contiguous() and x.shape == (n, pool.C)
    if out is None:
        out = (torch.zeros((n, 4), dtype=torch.int32, device="cuda"), torch.zeros_like(x),
               torch.zeros((1,), dtype=torch.int32, device="cuda"), torch.zeros((1,), dtype=torch.int32, device="cuda"))
    ws = _ws(dsvt_attn_pool_workspace_size(pool, n), ws)
    rc = lib().dsvt_attn_pool(C.byref(pool.struct), _ptr(coords), _ptr(x), n, _ptr(out[0]), _ptr(out[1]), _ptr(out[2]),
                              _ptr(ws), ws.numel(), _ptr(out[3]), _stream(stream))
    _check("dsvt_attn_pool", rc)
    return out


def dsvt_attn_pool_static(pool, coords, x, out, stream=None):
    """dsvt_attn_pool on the library's built-in scratch: no workspace, nothing allocated.  `out` = the caller's
    (out_coords [N,4] int32, out [N,C], n_out, status) tensors."""
    n = coords.shape[0]
    assert x.is_cuda and x.dtype == pool.dtype and x.is_contiguous() and x.shape == (n, pool.C)
    rc = lib().dsvt_attn_pool_static(C.byref(pool.struct), _ptr(coords), _ptr(x), n, _ptr(out[0]), _ptr(out[1]), _ptr(out[2]),
                                     _ptr(out[3]), _stream(stream))
    _check("dsvt_attn_pool_static", rc)
    return out


def dsvt_bev_scatter(coords, x, batch, grid, out=None, stream=None):
    """Dense channels-last map [batch, X, Y, Z, C] with every voxel's row at its cell, zeros elsewhere.
    Returns (out, status)."""
    n, c = x.shape
    assert x.is_cuda and x.is_contiguous() and coords.shape == (n, 4) and x.dtype in (torch.float32, torch.bfloat16)
    if out is None:
        out = torch.empty((batch, *grid, c), dtype=x.dtype, device="cuda")
    status = torch.zeros((1,), dtype=torch.int32, device="cuda")
    rc = lib().dsvt_bev_scatter(_ptr(coords), _ptr(x), n, c, DSVT_F32 if x.dtype == torch.float32 else DSVT_BF16, batch,
                                C.byref(I32x3(*grid)), _ptr(out), _ptr(status), _stream(stream))
    _check("dsvt_bev_scatter", rc)
    return out, status


def dsvt_vfe_workspace_size(cfg, n_points, max_voxels):
    b = C.c_size_t(0)
    _check("dsvt_vfe_workspace_size", lib().dsvt_vfe_workspace_size(C.byref(cfg), n_points, max_voxels, C.byref(b)))
    return b.value


class Vfe:
    """Configuration, weights and buffers of one dsvt_vfe call site: `max_points` points in, at most
    `max_voxels` voxels out.  w [C, f_in] and b [C] are float32 device tensors or None."""

    def __init__(self, grid, batch, range_min, voxel_size, f_in, C_out, dtype, max_points, max_voxels, w=None, b=None,
                 relu=False):
        self.w, self.b = w, b
        self.cfg = VfeCfg(I32x3(*grid), batch, F32x3(*range_min), F32x3(*voxel_size), f_in, C_out, _DT[dtype][0],
                          None if w is None else w.data_ptr(), None if b is None else b.data_ptr(), int(relu))
        self.max_points, self.max_voxels = max_points, max_voxels
        self.ws = torch.empty((dsvt_vfe_workspace_size(self.cfg, max_points, max_voxels),), dtype=torch.uint8, device="cuda")
        self.coords = torch.empty((max_voxels, 4), dtype=torch.int32, device="cuda")
        self.x = torch.empty((max_voxels, C_out), dtype=_DT[dtype][1], device="cuda")
        self.n_voxels = torch.zeros((1,), dtype=torch.int32, device="cuda")
        self.status = torch.zeros((1,), dtype=torch.int32, device="cuda")


def dsvt_vfe(vfe, points, point_batch=None, stream=None):
    """Encodes `points` [P, f_in] float32 (device) into vfe.coords / vfe.x / vfe.n_voxels."""
    n = points.shape[0]
    assert points.is_cuda and points.is_contiguous() and points.dtype == torch.float32 and n <= vfe.max_points
    assert points.shape[1] == vfe.cfg.f_in
    assert point_batch is None or (point_batch.is_cuda and point_batch.dtype == torch.int32 and point_batch.shape == (n,))
    rc = lib().dsvt_vfe(C.byref(vfe.cfg), _ptr(points), None if point_batch is None else _ptr(point_batch), n,
                        _ptr(vfe.coords), _ptr(vfe.x), _ptr(vfe.n_voxels), vfe.max_voxels, _ptr(vfe.ws), vfe.ws.numel(),
                        _ptr(vfe.status), _stream(stream))
    _check("dsvt_vfe", rc)
    return vfe


def prof_enable(max_launches):
    _check("dsvt_prof_enable", lib().dsvt_prof_enable(max_launches))


def prof_collect():
    """{kernel name: (total ms, launches)} for the launches recorded since prof_enable."""
    n = lib().dsvt_prof_kernel_count()
    ms, cnt = (C.c_float * n)(), (C.c_int32 * n)()
    _check("dsvt_prof_collect", lib().dsvt_prof_collect(ms, cnt, n))
    return {lib().dsvt_prof_kernel_name(k).decode(): (float(ms[k]), int(cnt[k])) for k in range(n)}
