"""ctypes binding of libpsconv.so: same names as the C ABI, argument marshalling only.

Tensors are passed as anything with a ``data_ptr()`` method (torch tensors) or as raw integer
device addresses.  The stream defaults to torch's current HIP stream.  Nothing here computes:
every step runs in the library's kernels, and the import fails loudly if the library is absent.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpsconv.so")

PS_OK, PS_EINVAL, PS_EUNSUPPORTED, PS_EHIP, PS_ESCRATCH = 0, -1, -2, -3, -4
PS_STATIC_SCRATCH_BYTES = 64 << 20
PS_F32, PS_BF16 = 0, 1


class ConvDesc(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("N", "C", "H", "W", "K", "R", "S", "stride", "pad", "dtype")]

    @classmethod
    def of(cls, shape, dtype: int = PS_F32) -> "ConvDesc":
        """From any object with N, C, H, W, K, R, S, stride, pad attributes."""
        return cls(shape.N, shape.C, shape.H, shape.W, shape.K, shape.R, shape.S,
                   shape.stride, shape.pad, dtype)


class Tile(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("kt", "mt", "ring", "c_split", "raster")]

    def as_tuple(self):
        return (self.kt, self.mt, self.ring, self.c_split, self.raster)

    def __repr__(self):
        return f"Tile(kt={self.kt}, mt={self.mt}, ring={self.ring}, c_split={self.c_split}, raster={self.raster})"


class LoopNest(ctypes.Structure):
    _fields_ = [("n_loops", ctypes.c_int32), ("extent", ctypes.c_int32 * 8)]


class ArrayRef(ctypes.Structure):
    """array[f_0][f_1]..., f_d = sum_l coef[d][l] * iter_l + offset[d]."""
    _fields_ = [("array", ctypes.c_int32), ("n_dims", ctypes.c_int32), ("is_write", ctypes.c_int32),
                ("elem_bytes", ctypes.c_int32), ("coef", (ctypes.c_int32 * 8) * 4), ("offset", ctypes.c_int32 * 4)]

    @classmethod
    def of(cls, array: int, coef, offset=None, is_write: bool = False, elem_bytes: int = 1):
        r = cls()
        r.array, r.n_dims, r.is_write, r.elem_bytes = array, len(coef), int(is_write), elem_bytes
        for d, row in enumerate(coef):
            for l, c in enumerate(row):
                r.coef[d][l] = c
            r.offset[d] = 0 if offset is None else offset[d]
        return r


class ReuseDep(ctypes.Structure):
    _fields_ = [("src_ref", ctypes.c_int32), ("tgt_ref", ctypes.c_int32), ("ws_min", ctypes.c_int64),
                ("ws_max", ctypes.c_int64)]


class Epilogue(ctypes.Structure):
    _fields_ = [("bias", ctypes.c_void_p), ("relu", ctypes.c_int32), ("out_dtype", ctypes.c_int32)]


class PsError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(f"{what}: {strerror(status)} (status {status})")


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()'). "
            "There is no CPU fallback.")
    # PyTorch ships a HIP runtime of its own.  Whichever copy is loaded first serves the whole process, and device
    # pointers and streams only mean something to the runtime that made them, so torch (the source of both here) has
    # to be loaded before the library binds to libamdhip64.
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    lib = ctypes.CDLL(LIB_PATH)
    dp = ctypes.POINTER(ConvDesc)
    tp = ctypes.POINTER(Tile)
    vp = ctypes.c_void_p
    i32p = ctypes.POINTER(ctypes.c_int32)
    sig = {
        "ps_out_dims": (ctypes.c_int, [dp, i32p, i32p]),
        "ps_blocked_in_bytes": (ctypes.c_size_t, [dp]),
        "ps_blocked_wt_bytes": (ctypes.c_size_t, [dp]),
        "ps_blocked_out_bytes": (ctypes.c_size_t, [dp]),
        "ps_nchw_to_blocked": (ctypes.c_int, [dp, vp, vp, vp]),
        "ps_blocked_to_nchw": (ctypes.c_int, [dp, vp, vp, vp]),
        "ps_kcrs_to_blocked": (ctypes.c_int, [dp, vp, vp, vp]),
        "ps_blocked_to_kcrs": (ctypes.c_int, [dp, vp, vp, vp]),
        "ps_blocked_to_nkpq": (ctypes.c_int, [dp, vp, vp, vp]),
        "ps_conv2d_fwd": (ctypes.c_int, [dp, vp, vp, vp, vp]),
        "ps_conv2d_fwd_tile": (ctypes.c_int, [dp, tp, vp, vp, vp, vp]),
        "ps_workspace_bytes": (ctypes.c_size_t, [dp, tp]),
        "ps_conv2d_fwd_ws": (ctypes.c_int, [dp, tp, vp, vp, vp, vp, ctypes.c_size_t, vp]),
        "ps_conv2d_fwd_static": (ctypes.c_int, [dp, tp, vp, vp, vp, vp]),
        "ps_conv2d_fwd_fused": (ctypes.c_int, [dp, tp, ctypes.POINTER(Epilogue), vp, vp, vp, vp, ctypes.c_size_t, vp]),
        "ps_tile_kernel": (ctypes.c_int, [dp, tp]),
        "ps_tile_pick": (ctypes.c_int, [dp, ctypes.c_int, ctypes.c_size_t, tp]),
        "ps_tile_cache_entries": (ctypes.c_size_t, []),
        "ps_tile_autotune": (ctypes.c_int, [dp, ctypes.c_int, vp, vp, vp, vp, ctypes.c_size_t, vp, tp, ctypes.POINTER(ctypes.c_double)]),
        "ps_tile_cost_ws_us": (ctypes.c_double, [dp, tp]),
        "ps_tile_select_ws": (ctypes.c_int, [dp, ctypes.c_size_t, tp, ctypes.POINTER(ctypes.c_double)]),
        "ps_probe_mfma": (ctypes.c_int, [ctypes.c_int, ctypes.c_int, vp, ctypes.POINTER(ctypes.c_double), vp]),
        "ps_tile_rank_ws": (ctypes.c_int, [dp, ctypes.c_size_t, ctypes.c_int, tp, ctypes.POINTER(ctypes.c_double)]),
        "ps_tile_count": (ctypes.c_int, [dp]),
        "ps_tile_get": (ctypes.c_int, [dp, ctypes.c_int, tp]),
        "ps_tile_valid": (ctypes.c_int, [dp, tp]),
        "ps_tile_cost_us": (ctypes.c_double, [dp, tp]),
        "ps_tile_select": (ctypes.c_int, [dp, tp, ctypes.POINTER(ctypes.c_double)]),
        "ps_strerror": (ctypes.c_char_p, [ctypes.c_int]),
        "ps_last_hip_error": (ctypes.c_char_p, []),
        "ps_reuse_working_sets": (ctypes.c_int, [ctypes.POINTER(LoopNest), ctypes.POINTER(ArrayRef), ctypes.c_int,
                                                 ctypes.POINTER(ReuseDep), ctypes.c_int]),
        "ps_reuse_assign": (ctypes.c_int, [ctypes.POINTER(ctypes.c_int64), ctypes.c_int, ctypes.POINTER(ctypes.c_int64),
                                           ctypes.c_int, ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_int64)]),
        "ps_reuse_cost": (ctypes.c_double, [ctypes.POINTER(ctypes.c_int64), ctypes.c_int, ctypes.c_int64,
                                            ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double)]),
        "ps_tile_reuse_levels": (ctypes.c_int, [dp, tp, ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_int64)]),
        "ps_tile_level_times_ws": (ctypes.c_int, [dp, tp, ctypes.POINTER(ctypes.c_double)]),
        "ps_tile_rank_dnn_scratch_bytes": (ctypes.c_size_t, [dp]),
        "ps_tile_rank_dnn": (ctypes.c_int, [dp, ctypes.c_size_t, ctypes.c_int, vp, ctypes.c_float, vp, ctypes.c_size_t,
                                            ctypes.c_int, tp, i32p, vp]),
        "ps_ranker_play": (ctypes.c_int, [vp, ctypes.c_int, vp, ctypes.c_float, vp, vp, vp]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    return lib


lib = _load()


def strerror(status: int) -> str:
    text = lib.ps_strerror(int(status)).decode()
    if status == PS_EHIP:
        text += ": " + ps_last_hip_error()
    return text


def ps_last_hip_error() -> str:
    return lib.ps_last_hip_error().decode()


def _ptr(t) -> int:
    if t is None:
        return 0
    return int(t.data_ptr()) if hasattr(t, "data_ptr") else int(t)


def _stream(stream) -> int:
    if stream is None:
        import torch
        return int(torch.cuda.current_stream().cuda_stream)
    return int(getattr(stream, "cuda_stream", stream))


def _check(status: int, what: str) -> None:
    if status != PS_OK:
        raise PsError(status, what)


def ps_out_dims(desc: ConvDesc) -> tuple[int, int]:
    P, Q = ctypes.c_int32(), ctypes.c_int32()
    _check(lib.ps_out_dims(ctypes.byref(desc), ctypes.byref(P), ctypes.byref(Q)), "ps_out_dims")
    return P.value, Q.value


def ps_blocked_in_bytes(desc: ConvDesc) -> int:
    return int(lib.ps_blocked_in_bytes(ctypes.byref(desc)))


def ps_blocked_wt_bytes(desc: ConvDesc) -> int:
    return int(lib.ps_blocked_wt_bytes(ctypes.byref(desc)))


def ps_blocked_out_bytes(desc: ConvDesc) -> int:
    return int(lib.ps_blocked_out_bytes(ctypes.byref(desc)))


def _transform(name: str):
    fn = getattr(lib, name)

    def call(desc: ConvDesc, src, dst, stream=None) -> None:
        _check(fn(ctypes.byref(desc), _ptr(src), _ptr(dst), _stream(stream)), name)

    call.__name__ = name
    return call


ps_nchw_to_blocked = _transform("ps_nchw_to_blocked")
ps_blocked_to_nchw = _transform("ps_blocked_to_nchw")
ps_kcrs_to_blocked = _transform("ps_kcrs_to_blocked")
ps_blocked_to_kcrs = _transform("ps_blocked_to_kcrs")
ps_blocked_to_nkpq = _transform("ps_blocked_to_nkpq")


def ps_conv2d_fwd(desc: ConvDesc, in_blk, wt_blk, out_blk, stream=None) -> None:
    _check(lib.ps_conv2d_fwd(ctypes.byref(desc), _ptr(in_blk), _ptr(wt_blk), _ptr(out_blk), _stream(stream)),
           "ps_conv2d_fwd")


def ps_conv2d_fwd_tile(desc: ConvDesc, tile: Tile, in_blk, wt_blk, out_blk, stream=None) -> None:
    _check(lib.ps_conv2d_fwd_tile(ctypes.byref(desc), ctypes.byref(tile), _ptr(in_blk), _ptr(wt_blk),
                                  _ptr(out_blk), _stream(stream)), "ps_conv2d_fwd_tile")


def ps_workspace_bytes(desc: ConvDesc, tile: Tile) -> int:
    return int(lib.ps_workspace_bytes(ctypes.byref(desc), ctypes.byref(tile)))


def ps_conv2d_fwd_ws(desc: ConvDesc, tile, in_blk, wt_blk, out_blk, workspace, workspace_bytes: int, stream=None) -> None:
    """tile=None lets the library pick among the tiles whose workspace fits."""
    tp = ctypes.byref(tile) if tile is not None else None
    _check(lib.ps_conv2d_fwd_ws(ctypes.byref(desc), tp, _ptr(in_blk), _ptr(wt_blk), _ptr(out_blk),
                                _ptr(workspace), int(workspace_bytes), _stream(stream)), "ps_conv2d_fwd_ws")


def ps_conv2d_fwd_static(desc: ConvDesc, tile, in_blk, wt_blk, out_blk, stream=None) -> None:
    """ps_conv2d_fwd_ws on the library's static scratch array (no allocation anywhere); tile=None lets it pick."""
    tp = ctypes.byref(tile) if tile is not None else None
    _check(lib.ps_conv2d_fwd_static(ctypes.byref(desc), tp, _ptr(in_blk), _ptr(wt_blk), _ptr(out_blk),
                                    _stream(stream)), "ps_conv2d_fwd_static")


def ps_conv2d_fwd_fused(desc: ConvDesc, tile, in_blk, wt_blk, out_blk, workspace=None, workspace_bytes: int = 0,
                        bias=None, relu: bool = False, out_dtype: int = PS_F32, stream=None) -> None:
    e = Epilogue(_ptr(bias) or None, int(relu), int(out_dtype))
    tp = ctypes.byref(tile) if tile is not None else None
    _check(lib.ps_conv2d_fwd_fused(ctypes.byref(desc), tp, ctypes.byref(e), _ptr(in_blk), _ptr(wt_blk), _ptr(out_blk),
                                   _ptr(workspace) or None, int(workspace_bytes), _stream(stream)), "ps_conv2d_fwd_fused")


KERNEL_NAMES = {0: "general", 1: "1x1 baked", 2: "1x1 pixel-stationary", 3: "3x3 baked", 5: "5x5 baked", 7: "tap-packed", 9: "3x3 patch"}


def ps_tile_kernel(desc: ConvDesc, tile: Tile) -> int:
    v = lib.ps_tile_kernel(ctypes.byref(desc), ctypes.byref(tile))
    if v < 0:
        raise PsError(v, "ps_tile_kernel")
    return v


def ps_tile_pick(desc: ConvDesc, with_workspace: bool = False, workspace_bytes: int = 0) -> Tile:
    """The tile the convolution calls run when none is passed (cached per descriptor inside the library)."""
    t = Tile()
    _check(lib.ps_tile_pick(ctypes.byref(desc), int(bool(with_workspace)), int(workspace_bytes), ctypes.byref(t)),
           "ps_tile_pick")
    return t


def ps_tile_autotune(desc: ConvDesc, k: int, in_blk, wt_blk, out_blk, workspace=None, workspace_bytes: int = 0,
                     stream=None) -> tuple[Tile, float, int]:
    """Runs the model's k best tiles on the given tensors and makes the fastest the descriptor's pick; returns
    (tile, microseconds per launch, candidates timed).  Waits for the stream."""
    t, us = Tile(), ctypes.c_double()
    n = lib.ps_tile_autotune(ctypes.byref(desc), int(k), _ptr(in_blk), _ptr(wt_blk), _ptr(out_blk), _ptr(workspace) or None,
                             int(workspace_bytes), _stream(stream), ctypes.byref(t), ctypes.byref(us))
    if n < 0:
        raise PsError(n, "ps_tile_autotune")
    return t, us.value, n


def ps_tile_cache_entries() -> int:
    return int(lib.ps_tile_cache_entries())


def ps_tile_cost_ws_us(desc: ConvDesc, tile: Tile) -> float:
    return float(lib.ps_tile_cost_ws_us(ctypes.byref(desc), ctypes.byref(tile)))


def ps_tile_select_ws(desc: ConvDesc, workspace_bytes: int) -> tuple[Tile, float]:
    t, us = Tile(), ctypes.c_double()
    _check(lib.ps_tile_select_ws(ctypes.byref(desc), int(workspace_bytes), ctypes.byref(t), ctypes.byref(us)),
           "ps_tile_select_ws")
    return t, us.value


def ps_probe_mfma(dtype: int, iters: int, sink, stream=None) -> float:
    """Launches the MFMA-only loop; returns the FLOP it performs (time it with events on the stream)."""
    flop = ctypes.c_double()
    _check(lib.ps_probe_mfma(int(dtype), int(iters), _ptr(sink), ctypes.byref(flop), _stream(stream)), "ps_probe_mfma")
    return flop.value


def ps_tile_rank_ws(desc: ConvDesc, workspace_bytes: int, k: int) -> list[tuple[Tile, float]]:
    tiles, us = (Tile * k)(), (ctypes.c_double * k)()
    n = lib.ps_tile_rank_ws(ctypes.byref(desc), int(workspace_bytes), int(k), tiles, us)
    if n < 0:
        raise PsError(n, "ps_tile_rank_ws")
    return [(Tile(tiles[i].kt, tiles[i].mt, tiles[i].ring, tiles[i].c_split, tiles[i].raster), us[i]) for i in range(n)]


def ps_tile_count(desc: ConvDesc) -> int:
    n = lib.ps_tile_count(ctypes.byref(desc))
    if n < 0:
        raise PsError(n, "ps_tile_count")
    return n


def ps_tile_get(desc: ConvDesc, idx: int) -> Tile:
    t = Tile()
    _check(lib.ps_tile_get(ctypes.byref(desc), int(idx), ctypes.byref(t)), "ps_tile_get")
    return t


def ps_tile_valid(desc: ConvDesc, tile: Tile) -> bool:
    return lib.ps_tile_valid(ctypes.byref(desc), ctypes.byref(tile)) == PS_OK


def ps_tile_cost_us(desc: ConvDesc, tile: Tile) -> float:
    return float(lib.ps_tile_cost_us(ctypes.byref(desc), ctypes.byref(tile)))


def ps_tile_select(desc: ConvDesc) -> tuple[Tile, float]:
    t, us = Tile(), ctypes.c_double()
    _check(lib.ps_tile_select(ctypes.byref(desc), ctypes.byref(t), ctypes.byref(us)), "ps_tile_select")
    return t, us.value


def ps_reuse_working_sets(extents, refs) -> list[tuple[int, int, int, int]]:
    """Algorithm 1 on a rectangular nest: [(src_ref, tgt_ref, ws_min, ws_max), ...] for every dependence."""
    nest = LoopNest()
    nest.n_loops = len(extents)
    for l, e in enumerate(extents):
        nest.extent[l] = e
    arr = (ArrayRef * len(refs))(*refs)
    n = lib.ps_reuse_working_sets(ctypes.byref(nest), arr, len(refs), None, 0)
    if n < 0:
        raise PsError(n, "ps_reuse_working_sets")
    out = (ReuseDep * max(n, 1))()
    n = lib.ps_reuse_working_sets(ctypes.byref(nest), arr, len(refs), out, n)
    if n < 0:
        raise PsError(n, "ps_reuse_working_sets")
    return [(out[i].src_ref, out[i].tgt_ref, out[i].ws_min, out[i].ws_max) for i in range(n)]


def ps_reuse_assign(ws, cache_sizes) -> tuple[list[int], int]:
    """Algorithm 2: ([WS per cache level], WS served from memory)."""
    ws, cache_sizes = list(ws), list(cache_sizes)
    w = (ctypes.c_int64 * max(len(ws), 1))(*ws)
    c = (ctypes.c_int64 * max(len(cache_sizes), 1))(*cache_sizes)
    lvl = (ctypes.c_int64 * max(len(cache_sizes), 1))()
    mem = ctypes.c_int64()
    _check(lib.ps_reuse_assign(w, len(ws), c, len(cache_sizes), lvl, ctypes.byref(mem)), "ps_reuse_assign")
    return [lvl[i] for i in range(len(cache_sizes))], mem.value


def ps_reuse_cost(level_ws, mem_ws: int, lat, bw) -> float:
    """Eq. 1; lat and bw carry one entry per cache level and a last one for memory."""
    n = len(level_ws)
    if len(lat) != n + 1 or len(bw) != n + 1:
        raise PsError(PS_EINVAL, "ps_reuse_cost")
    c = lib.ps_reuse_cost((ctypes.c_int64 * max(n, 1))(*level_ws), n, int(mem_ws),
                          (ctypes.c_double * (n + 1))(*lat), (ctypes.c_double * (n + 1))(*bw))
    if c < 0:
        raise PsError(PS_EINVAL, "ps_reuse_cost")
    return c


PS_RANKER_STATS = 4
PS_RANKER_LEVELS = 3
PS_RANKER_PARAMS = 3338
PS_RANKER_MAX_VARIANTS = 8192
PS_RANKER_WORKING_SETS, PS_RANKER_LEVEL_TIMES = 0, 1


def ps_tile_reuse_levels(desc: ConvDesc, tile: Tile) -> tuple[list[int], int]:
    """Working-set sizes (bytes) of a candidate tile at registers+LDS, L2 and Infinity Cache, and what is left to
    memory (Algorithms 1 and 2 on the tile's workgroup-level loop nest)."""
    lvl = (ctypes.c_int64 * PS_RANKER_LEVELS)()
    mem = ctypes.c_int64()
    _check(lib.ps_tile_reuse_levels(ctypes.byref(desc), ctypes.byref(tile), lvl, ctypes.byref(mem)),
           "ps_tile_reuse_levels")
    return [lvl[i] for i in range(PS_RANKER_LEVELS)], mem.value


def ps_tile_level_times_ws(desc: ConvDesc, tile: Tile) -> list[float]:
    """The four parts of the tile model's cost (us): matrix cores, traffic into the compute units, traffic beyond
    L2, launches and extra passes."""
    out = (ctypes.c_double * PS_RANKER_STATS)()
    _check(lib.ps_tile_level_times_ws(ctypes.byref(desc), ctypes.byref(tile), out), "ps_tile_level_times_ws")
    return [out[i] for i in range(PS_RANKER_STATS)]


def ps_ranker_play(stats, n: int, params, theta: float, wins, probs=None, stream=None) -> None:
    """The tournament of Section 4.2.2: stats float32 [n][4], params float32 [PS_RANKER_PARAMS], wins int32 [n],
    probs float32 [n][n][2] or None -- all device tensors."""
    _check(lib.ps_ranker_play(_ptr(stats), n, _ptr(params), theta, _ptr(wins), None if probs is None else _ptr(probs),
                              _stream(stream)), "ps_ranker_play")


def ps_tile_rank_dnn_scratch_bytes(desc: ConvDesc) -> int:
    return int(lib.ps_tile_rank_dnn_scratch_bytes(ctypes.byref(desc)))


def ps_tile_rank_dnn(desc: ConvDesc, workspace_bytes: int, stats_kind: int, params, theta: float, scratch,
                     scratch_bytes: int, k: int, stream=None) -> list[tuple[Tile, int]]:
    """The k candidates with the most tournament wins, [(tile, wins), ...]; params and scratch are device tensors.
    Waits for the stream."""
    tiles = (Tile * k)()
    wins = (ctypes.c_int32 * k)()
    n = lib.ps_tile_rank_dnn(ctypes.byref(desc), workspace_bytes, stats_kind, _ptr(params), theta, _ptr(scratch),
                             scratch_bytes, k, tiles, wins, _stream(stream))
    if n < 0:
        raise PsError(n, "ps_tile_rank_dnn")
    return [(Tile(*tiles[i].as_tuple()), int(wins[i])) for i in range(n)]
