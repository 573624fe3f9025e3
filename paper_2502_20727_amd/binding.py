"""ctypes binding of the SPD C ABI (include/spd.h, include/spd_testing.h): same names, argument marshalling only.

Every step of the decoder-block path runs inside the HIP library; this module turns NumPy
arrays / torch tensors / Python ints into the pointers and sizes the C calls take and turns
error codes into exceptions.  PyTorch appears only as the owner of device memory and of
the stream.  If the HIP library cannot be loaded this module raises: there is no fallback.
"""
from __future__ import annotations

import ctypes as C
from typing import Dict, List, Optional, Sequence

import numpy as np

from . import build
from .workloads import Workload

SPD_F32, SPD_BF16 = 0, 1
SPD_OK, SPD_EINVAL, SPD_EUNSUPPORTED, SPD_EHIP, SPD_ETOOBIG = 0, -1, -2, -3, -4
SPD_STATIC_WORKSPACE_BYTES = 64 << 20
SPD_ALL_RANKS = -1
SPD_MAX_BATCH = 64


class SpdError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        detail = ""
        if code == SPD_EHIP:
            msg = lib().spd_last_hip_error()
            detail = f": {msg.decode()}" if msg else ""
        super().__init__(f"{where}: {strerror(code)} ({code}){detail}")


class spd_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("hidden", "n_q_heads", "n_kv_heads", "head_dim", "ffn", "n_layers",
                                         "tp_degree", "dtype", "max_batch", "max_ctx", "max_tokens")] + \
               [("rms_eps", C.c_float), ("rope_base", C.c_float), ("act_split", C.c_int32), ("o_bias", C.c_int32)]


SPD_SPLIT_AUTO, SPD_SPLIT_ALWAYS, SPD_SPLIT_NEVER = 0, 1, 2
SPD_TIER_TP, SPD_TIER_ISB, SPD_TIER_SB, SPD_TIER_ESB = 0, 1, 2, 3


class spd_sizes(C.Structure):
    _fields_ = [("weight_bytes", C.c_size_t), ("kv_bytes", C.c_size_t), ("workspace_bytes", C.c_size_t)]


_FP = C.POINTER(C.c_float)


class spd_layer_weights(C.Structure):
    _fields_ = [(n, _FP) for n in ("wq", "wk", "wv", "wo", "wg", "wu", "wd", "g1", "g2")] + \
               [(n, C.c_int64) for n in ("ld_q", "ld_k", "ld_v", "ld_o", "ld_g", "ld_u", "ld_d")] + [("bo", _FP)]


class spd_taps(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("q", "attn", "y", "u")]


_lib = None

_PROTOS = {
    "spd_create": (C.c_int, [C.POINTER(spd_config), C.POINTER(C.c_void_p)]),
    "spd_destroy": (None, [C.c_void_p]),
    "spd_get_config": (C.c_int, [C.c_void_p, C.POINTER(spd_config)]),
    "spd_get_sizes": (C.c_int, [C.c_void_p, C.POINTER(spd_sizes)]),
    "spd_last_hip_error": (C.c_char_p, []),
    "spd_strerror": (C.c_char_p, [C.c_int]),
    "spd_rank_q_heads": (C.c_int, [C.c_void_p, C.c_int32, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]),
    "spd_rank_kv_heads": (C.c_int, [C.c_void_p, C.c_int32, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]),
    "spd_rank_ffn_cols": (C.c_int, [C.c_void_p, C.c_int32, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]),
    "spd_sync_count": (C.c_int64, [C.c_void_p, C.c_void_p]),
    "spd_mask_from_sensitivity": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32, C.c_double, C.c_double, C.c_void_p,
                                            C.c_void_p]),
    "spd_pack_shard": (C.c_int, [C.c_void_p, C.c_int32, C.POINTER(spd_layer_weights), C.c_void_p]),
    "spd_pack_shard_grouped": (C.c_int, [C.c_void_p, C.c_int32, C.POINTER(spd_layer_weights), C.c_void_p, C.c_void_p,
                                         C.c_void_p]),
    "spd_pack_shard_local": (C.c_int, [C.c_void_p, C.POINTER(spd_layer_weights), C.c_void_p]),
    "spd_unpack_shard": (C.c_int, [C.c_void_p, C.c_void_p, C.POINTER(spd_layer_weights)]),
    "spd_kv_pack": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p]),
    "spd_kv_unpack": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]),
    "spd_workspace_init": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p]),
    "spd_rank_sum": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int64, C.c_void_p, C.c_void_p]),
    "spd_block_forward": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                                    C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                    C.c_void_p, C.c_void_p, C.POINTER(spd_taps)]),
    "spd_block_forward_static": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                                           C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                           C.c_void_p, C.POINTER(spd_taps)]),
    "spd_model_forward": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                    C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                    C.c_void_p, C.POINTER(C.c_int64)]),
    "spd_model_forward_staged": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                           C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                           C.c_void_p, C.POINTER(C.c_int64), C.c_uint32, C.c_void_p, C.c_void_p]),
    "spd_stage_timer_create": (C.c_int, [C.c_int32, C.c_int32, C.POINTER(C.c_void_p)]),
    "spd_stage_timer_read": (C.c_int, [C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_double), C.POINTER(C.c_double)]),
    "spd_stage_timer_destroy": (None, [C.c_void_p]),
    "spd_mfma_probe": (C.c_int, [C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_double)]),
    "spd_read_probe": (C.c_int, [C.c_void_p, C.c_size_t, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.POINTER(C.c_double)]),
    "spd_gemm_launch_size": (C.c_int, [C.c_int32]),
    "spd_gemm_tile_of": (C.c_int, [C.c_int32] * 7 + [C.POINTER(C.c_int32), C.POINTER(C.c_int32)]),
}
EXPORTS = tuple(_PROTOS)
STAGES = {"prep": 0, "qkv": 1, "attn": 2, "o": 3, "gateup": 4, "down": 5}
SPD_ALL_STAGES = (1 << len(STAGES)) - 1
SPD_STAGE_EMPTY = len(STAGES)


def lib():
    """The loaded HIP library.  Raises if it is missing and cannot be built."""
    global _lib
    if _lib is None:
        path = build.ensure_hip()
        # PyTorch ships its own HIP runtime.  The library must bind to the same one as the tensors it
        # is handed, so torch (when installed) is imported before the library is loaded: loaded the
        # other way round, the process holds two runtimes and this library's calls see no device.
        try:
            import torch  # noqa: F401
        except ImportError:
            pass
        l = C.CDLL(path)
        for name, (res, args) in _PROTOS.items():
            fn = getattr(l, name)          # AttributeError if the symbol is not exported
            fn.restype = res
            fn.argtypes = args
        _lib = l
    return _lib


def strerror(code: int) -> str:
    return lib().spd_strerror(code).decode()


def _check(code: int, where: str) -> None:
    if code != SPD_OK:
        raise SpdError(code, where)


def _ptr(x) -> Optional[int]:
    """Address of a torch tensor / NumPy array / raw int; None stays NULL."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if isinstance(x, np.ndarray):
        assert x.flags.c_contiguous
        return x.ctypes.data
    assert x.is_contiguous()
    return x.data_ptr()


def _i32(values: Sequence[int]):
    arr = (C.c_int32 * max(len(values), 1))(*[int(v) for v in values])
    return arr


# --------------------------------------------------------------------------- host-only calls

def make_config(w: Workload, max_batch: Optional[int] = None, max_ctx: Optional[int] = None,
                max_tokens: Optional[int] = None, act_split: int = 0, o_bias: int = 0) -> spd_config:
    mb = max_batch if max_batch is not None else w.batch
    mc = max_ctx if max_ctx is not None else (w.ctx + 31) // 32 * 32
    mt = max_tokens if max_tokens is not None else max(w.batch * w.q_len, mb)
    return spd_config(w.hidden, w.n_q_heads, w.n_kv_heads, w.head_dim, w.ffn, w.n_layers, w.tp, w.dtype,
                      mb, mc, mt, w.rms_eps, w.rope_base, act_split, o_bias)


def spd_create(cfg: spd_config) -> int:
    out = C.c_void_p()
    _check(lib().spd_create(C.byref(cfg), C.byref(out)), "spd_create")
    return out.value


def spd_destroy(ctx: int) -> None:
    lib().spd_destroy(ctx)


def spd_get_sizes(ctx: int) -> spd_sizes:
    s = spd_sizes()
    _check(lib().spd_get_sizes(ctx, C.byref(s)), "spd_get_sizes")
    return s


def spd_get_config(ctx: int) -> spd_config:
    c = spd_config()
    _check(lib().spd_get_config(ctx, C.byref(c)), "spd_get_config")
    return c


def _range_call(fn, ctx, rank):
    a, b = C.c_int32(), C.c_int32()
    _check(fn(ctx, rank, C.byref(a), C.byref(b)), fn.__name__)
    return a.value, b.value


def spd_rank_q_heads(ctx: int, rank: int):
    return _range_call(lib().spd_rank_q_heads, ctx, rank)


def spd_rank_kv_heads(ctx: int, rank: int):
    return _range_call(lib().spd_rank_kv_heads, ctx, rank)


def spd_rank_ffn_cols(ctx: int, rank: int):
    return _range_call(lib().spd_rank_ffn_cols, ctx, rank)


def spd_sync_count(ctx: int, mask: Sequence[int]) -> int:
    m = np.ascontiguousarray(mask, dtype=np.uint8)
    n = lib().spd_sync_count(ctx, m.ctypes.data)
    if n < 0:
        raise SpdError(int(n), "spd_sync_count")
    return int(n)


def spd_mask_from_sensitivity(sensitivity: Sequence[float], n_spd: int, tau1: float, tau2: float):
    """Returns (mask, tier), two lists of n_layers ints."""
    s = np.ascontiguousarray(sensitivity, dtype=np.float64)
    mask = np.zeros(s.size, dtype=np.uint8)
    tier = np.zeros(s.size, dtype=np.uint8)
    _check(lib().spd_mask_from_sensitivity(s.ctypes.data if s.size else None, s.size, int(n_spd), float(tau1),
                                           float(tau2), mask.ctypes.data, tier.ctypes.data),
           "spd_mask_from_sensitivity")
    return mask.tolist(), tier.tolist()


def _weights_struct(W: Dict[str, np.ndarray]) -> spd_layer_weights:
    s = spd_layer_weights()
    for name in ("wq", "wk", "wv", "wo", "wg", "wu", "wd", "g1", "g2"):
        a = W[name]
        assert a.dtype == np.float32 and a.flags.c_contiguous, name
        setattr(s, name, a.ctypes.data_as(_FP))
    for name, ld in (("wq", "ld_q"), ("wk", "ld_k"), ("wv", "ld_v"), ("wo", "ld_o"), ("wg", "ld_g"),
                     ("wu", "ld_u"), ("wd", "ld_d")):
        setattr(s, ld, W[name].shape[1])
    if W.get("bo") is not None:          # bias of the output projection (block with bias)
        assert W["bo"].dtype == np.float32 and W["bo"].flags.c_contiguous
        s.bo = W["bo"].ctypes.data_as(_FP)
    return s


def spd_pack_shard(ctx: int, rank: int, dense: Dict[str, np.ndarray], out: Optional[np.ndarray] = None) -> np.ndarray:
    if out is None:
        out = np.empty(spd_get_sizes(ctx).weight_bytes, dtype=np.uint8)
    s = _weights_struct(dense)
    _check(lib().spd_pack_shard(ctx, rank, C.byref(s), out.ctypes.data), "spd_pack_shard")
    return out


def spd_pack_shard_grouped(ctx: int, rank: int, dense: Dict[str, np.ndarray], kv_heads: Optional[Sequence[int]],
                           mlp_of_rank: Optional[Sequence[int]], out: Optional[np.ndarray] = None) -> np.ndarray:
    if out is None:
        out = np.empty(spd_get_sizes(ctx).weight_bytes, dtype=np.uint8)
    s = _weights_struct(dense)
    kh = None if kv_heads is None else np.ascontiguousarray(kv_heads, dtype=np.int32)
    mr = None if mlp_of_rank is None else np.ascontiguousarray(mlp_of_rank, dtype=np.int32)
    _check(lib().spd_pack_shard_grouped(ctx, rank, C.byref(s), None if kh is None else kh.ctypes.data,
                                        None if mr is None else mr.ctypes.data, out.ctypes.data), "spd_pack_shard_grouped")
    return out


def spd_pack_shard_local(ctx: int, shard: Dict[str, np.ndarray], out: Optional[np.ndarray] = None) -> np.ndarray:
    if out is None:
        out = np.empty(spd_get_sizes(ctx).weight_bytes, dtype=np.uint8)
    s = _weights_struct(shard)
    _check(lib().spd_pack_shard_local(ctx, C.byref(s), _ptr(out)), "spd_pack_shard_local")
    return out


def spd_unpack_shard(ctx: int, packed: np.ndarray, shapes: Dict[str, tuple]) -> Dict[str, np.ndarray]:
    out = {k: np.zeros(v, dtype=np.float32) for k, v in shapes.items()}
    s = _weights_struct(out)
    _check(lib().spd_unpack_shard(ctx, packed.ctypes.data, C.byref(s)), "spd_unpack_shard")
    return out


def spd_kv_pack(ctx: int, k: np.ndarray, v: np.ndarray, cache_host: np.ndarray) -> None:
    assert k.dtype == np.float32 and v.dtype == np.float32 and k.shape == v.shape
    batch, _, n_pos, _ = k.shape
    _check(lib().spd_kv_pack(ctx, _ptr(np.ascontiguousarray(k)), _ptr(np.ascontiguousarray(v)), batch, n_pos,
                             cache_host.ctypes.data), "spd_kv_pack")


def spd_kv_unpack(ctx: int, cache_host: np.ndarray, batch: int, n_pos: int, kv_heads: int, head_dim: int):
    k = np.zeros((batch, kv_heads, n_pos, head_dim), dtype=np.float32)
    v = np.zeros_like(k)
    _check(lib().spd_kv_unpack(ctx, cache_host.ctypes.data, batch, n_pos, k.ctypes.data, v.ctypes.data), "spd_kv_unpack")
    return k, v


# --------------------------------------------------------------------------- device calls

def _stream_ptr(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def spd_workspace_init(ctx: int, workspace, stream=None) -> None:
    _check(lib().spd_workspace_init(ctx, _ptr(workspace), _stream_ptr(stream)), "spd_workspace_init")


def spd_rank_sum(ctx: int, base, slots, n_slots: int, n_elems: int, out, stream=None) -> None:
    _check(lib().spd_rank_sum(ctx, _ptr(base), _ptr(slots), n_slots, n_elems, _ptr(out), _stream_ptr(stream)),
           "spd_rank_sum")


def spd_block_forward(ctx: int, layer: int, spd_flag: int, rank: int, packed_weights, kv_cache,
                      positions: Sequence[int], batch: int, q_len: int, x_in, slots, x_out, workspace,
                      stream=None, taps: Optional[Dict[str, object]] = None) -> None:
    t = None
    if taps:
        t = spd_taps(*[_ptr(taps.get(n)) for n in ("q", "attn", "y", "u")])
    _check(lib().spd_block_forward(ctx, layer, spd_flag, rank, _ptr(packed_weights), _ptr(kv_cache),
                                   C.cast(_i32(positions), C.c_void_p), batch, q_len, _ptr(x_in), _ptr(slots),
                                   _ptr(x_out), _ptr(workspace), _stream_ptr(stream),
                                   C.byref(t) if t is not None else None), "spd_block_forward")


def spd_block_forward_static(ctx: int, layer: int, spd_flag: int, rank: int, packed_weights, kv_cache,
                             positions: Sequence[int], batch: int, q_len: int, x_in, slots, x_out,
                             stream=None, taps: Optional[Dict[str, object]] = None) -> None:
    t = None
    if taps:
        t = spd_taps(*[_ptr(taps.get(n)) for n in ("q", "attn", "y", "u")])
    _check(lib().spd_block_forward_static(ctx, layer, spd_flag, rank, _ptr(packed_weights), _ptr(kv_cache),
                                          C.cast(_i32(positions), C.c_void_p), batch, q_len, _ptr(x_in), _ptr(slots),
                                          _ptr(x_out), _stream_ptr(stream), C.byref(t) if t is not None else None),
           "spd_block_forward_static")


def spd_model_forward(ctx: int, spd_mask: Sequence[int], rank: int, layer_weights: Sequence, layer_kv: Sequence,
                      positions: Sequence[int], batch: int, q_len: int, x_in, slots, x_out, workspace,
                      stream=None) -> int:
    mask = np.ascontiguousarray(spd_mask, dtype=np.uint8)
    n = len(layer_weights)
    wp = (C.c_void_p * n)(*[_ptr(t) for t in layer_weights])
    kp = (C.c_void_p * n)(*[_ptr(t) for t in layer_kv])
    syncs = C.c_int64(0)
    _check(lib().spd_model_forward(ctx, mask.ctypes.data, rank, C.cast(wp, C.c_void_p), C.cast(kp, C.c_void_p),
                                   C.cast(_i32(positions), C.c_void_p), batch, q_len, _ptr(x_in), _ptr(slots),
                                   _ptr(x_out), _ptr(workspace), _stream_ptr(stream), C.byref(syncs)),
           "spd_model_forward")
    return syncs.value


def spd_model_forward_staged(ctx: int, spd_mask: Sequence[int], rank: int, layer_weights: Sequence, layer_kv: Sequence,
                             positions: Sequence[int], batch: int, q_len: int, x_in, slots, x_out, workspace,
                             stage_mask: int = SPD_ALL_STAGES, timer: Optional[int] = None, stream=None,
                             layer_out=None) -> int:
    mask = np.ascontiguousarray(spd_mask, dtype=np.uint8)
    n = len(layer_weights)
    wp = (C.c_void_p * n)(*[_ptr(t) for t in layer_weights])
    kp = (C.c_void_p * n)(*[_ptr(t) for t in layer_kv])
    syncs = C.c_int64(0)
    _check(lib().spd_model_forward_staged(ctx, mask.ctypes.data, rank, C.cast(wp, C.c_void_p), C.cast(kp, C.c_void_p),
                                          C.cast(_i32(positions), C.c_void_p), batch, q_len, _ptr(x_in), _ptr(slots),
                                          _ptr(x_out), _ptr(workspace), _stream_ptr(stream), C.byref(syncs),
                                          int(stage_mask), timer, _ptr(layer_out)),
           "spd_model_forward_staged")
    return syncs.value


def spd_stage_timer_create(stage: int, max_records: int) -> int:
    out = C.c_void_p()
    _check(lib().spd_stage_timer_create(stage, max_records, C.byref(out)), "spd_stage_timer_create")
    return out.value


def spd_stage_timer_read(timer: int):
    """(launches timed, mean microseconds, min microseconds) since the last read."""
    n, mean, mn = C.c_int32(), C.c_double(), C.c_double()
    _check(lib().spd_stage_timer_read(timer, C.byref(n), C.byref(mean), C.byref(mn)), "spd_stage_timer_read")
    return n.value, mean.value, mn.value


def spd_stage_timer_destroy(timer: int) -> None:
    lib().spd_stage_timer_destroy(timer)


SPD_MFMA_PROBE_SCRATCH_BYTES = 256 * 512 * 4 + 16


def spd_mfma_probe(iters: int, random_data: bool, scratch, stream=None):
    """(TFLOP/s, shader MHz) of register-resident 16x16x32 fp16 MFMAs over a full grid; `scratch` is a device
    tensor of at least SPD_MFMA_PROBE_SCRATCH_BYTES."""
    assert scratch.is_cuda and scratch.numel() * scratch.element_size() >= SPD_MFMA_PROBE_SCRATCH_BYTES
    tf, mhz = C.c_double(), C.c_double()
    _check(lib().spd_mfma_probe(iters, 1 if random_data else 0, scratch.data_ptr(), _stream_ptr(stream), C.byref(tf),
                                C.byref(mhz)), "spd_mfma_probe")
    return tf.value, mhz.value


def spd_read_probe(buf, chunk_bytes: int, n_chunks: int, reps: int, sink, stream=None) -> float:
    """Mean microseconds per launch of a kernel that only reads chunk_bytes (device tensors `buf`, `sink`)."""
    assert buf.is_cuda and buf.numel() * buf.element_size() >= chunk_bytes * n_chunks and sink.is_cuda
    us = C.c_double()
    _check(lib().spd_read_probe(buf.data_ptr(), chunk_bytes, n_chunks, reps, sink.data_ptr(), _stream_ptr(stream), C.byref(us)),
           "spd_read_probe")
    return us.value


def spd_gemm_launch_size(n_tiles: int) -> int:
    """Workgroups launched for `n_tiles` tiles of the GEMM's tile order."""
    n = lib().spd_gemm_launch_size(n_tiles)
    if n < 0:
        _check(n, "spd_gemm_launch_size")
    return n


def spd_gemm_tile_of(TN: int, TM: int, rn: int, rm: int, tile0: int, n_tiles: int, b: int):
    """(tn, tm) of the tile that workgroup `b` takes, or None for a spare workgroup."""
    tn, tm = C.c_int32(), C.c_int32()
    rc = lib().spd_gemm_tile_of(TN, TM, rn, rm, tile0, n_tiles, b, C.byref(tn), C.byref(tm))
    if rc == 1:
        return None
    _check(rc, "spd_gemm_tile_of")
    return tn.value, tm.value


# --------------------------------------------------------------------------- device-memory plumbing

class DeviceShard:
    """Device buffers (torch tensors) of one rank, or of all ranks back to back, for a workload.

    Holds memory only; every computation goes through the spd_* calls above.
    """

    def __init__(self, w: Workload, ranks: Sequence[int], device, max_ctx: Optional[int] = None,
                 max_tokens: Optional[int] = None, max_batch: Optional[int] = None, act_split: int = 0,
                 o_bias: int = 0):
        import torch
        self.torch = torch
        self.w = w
        self.ranks = list(ranks)
        self.device = device
        self.cfg = make_config(w, max_batch=max_batch, max_ctx=max_ctx, max_tokens=max_tokens, act_split=act_split,
                               o_bias=o_bias)
        self.ctx = spd_create(self.cfg)
        self.sizes = spd_get_sizes(self.ctx)
        nr = len(self.ranks)
        u8 = torch.uint8
        self.weights = [torch.empty(nr * self.sizes.weight_bytes, dtype=u8, device=device) for _ in range(w.n_layers)]
        self.kv = [torch.zeros(nr * self.sizes.kv_bytes, dtype=u8, device=device) for _ in range(w.n_layers)]
        self.workspace = torch.zeros(self.sizes.workspace_bytes, dtype=u8, device=device)
        spd_workspace_init(self.ctx, self.workspace)

    def close(self):
        if self.ctx:
            spd_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def load_layer(self, layer: int, shards: List[Dict[str, np.ndarray]]) -> None:
        """Pack (host) and upload the given ranks' shards of one layer."""
        torch = self.torch
        wb = self.sizes.weight_bytes
        host = np.empty(len(shards) * wb, dtype=np.uint8)
        for i, s in enumerate(shards):
            spd_pack_shard_local(self.ctx, s, host[i * wb:(i + 1) * wb])
        self.weights[layer].copy_(torch.from_numpy(host))

    def load_kv(self, layer: int, kvs: List[tuple]) -> None:
        """kvs[i] = (k, v) natural-layout prefill of rank i: [batch, kv, n_pos, d] fp32."""
        torch = self.torch
        kb = self.sizes.kv_bytes
        host = np.zeros(len(kvs) * kb, dtype=np.uint8)
        for i, (k, v) in enumerate(kvs):
            spd_kv_pack(self.ctx, k, v, host[i * kb:(i + 1) * kb])
        self.kv[layer].copy_(torch.from_numpy(host))

    def read_kv(self, layer: int, rank_index: int, batch: int, n_pos: int):
        kb = self.sizes.kv_bytes
        host = self.kv[layer][rank_index * kb:(rank_index + 1) * kb].cpu().numpy()
        return spd_kv_unpack(self.ctx, host, batch, n_pos, self.w.kv_per_rank, self.w.head_dim)

    def rank_arg(self) -> int:
        return SPD_ALL_RANKS if len(self.ranks) > 1 else self.ranks[0]
