"""ctypes binding of libzipmoe (include/zipmoe.h): argument marshalling only.

Every step of the decode path runs in the library's HIP kernels; PyTorch is used
by callers for device memory and streams.  The library must have been built
(``python -m paper_2601_21198_amd.build`` or ``__graft_entry__.build()``);
loading fails loudly otherwise -- there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence, Tuple

import numpy as np

from .build import LIB_PATH

OK, E_ARG, E_SIZE, E_FORMAT, E_HIP, E_NOMEM = 0, -1, -2, -3, -4, -5
MAX_CODE_LEN = 12
TILE_VALUES = 512
MODE_CODED, MODE_RAW = 0, 1
STAGING_BYTES = 32 << 20
STORES_AUTO, STORES_CACHED, STORES_STREAMING = 0, 1, 2

EXPORTS = ("zm_version", "zm_strerror", "zm_exponent_histogram", "zm_build_codebook", "zm_encode_bound",
           "zm_encode", "zm_blob_info", "zm_validate_blob", "zm_decode_experts", "zm_decode_experts_stores", "zm_decode_launch_shapes", "zm_decode_tensors", "zm_decode_host_tensors",
           "zm_layer_arena_bytes", "zm_layer_create", "zm_layer_tensor_info", "zm_layer_decode", "zm_layer_destroy",
           "zm_decode_exponents_host", "zm_recover", "zm_mover_probe", "zm_cache_dispatch", "zm_cache_arena_bytes", "zm_cache_image_bytes",
           "zm_cache_pack_expert", "zm_cache_create",
           "zm_cache_fetch", "zm_cache_pool_of", "zm_cache_destroy", "zm_plan_selection_probabilities",
           "zm_plan_hit_distribution", "zm_plan_makespan", "zm_plan_expected_makespan", "zm_plan_pools",
           "zm_sched_build", "zm_sched_simulate", "zm_sched_lower_bounds")
POOL_FULL, POOL_COMPRESSED, POOL_SM, POOL_E, POOL_NONE = 0, 1, 2, 3, 4


class TensorInfo(ctypes.Structure):
    """zm_tensor_info"""
    _fields_ = [("n_values", ctypes.c_uint64), ("blob_size", ctypes.c_uint64), ("lut_offset", ctypes.c_uint64),
                ("table_offset", ctypes.c_uint64), ("sm_offset", ctypes.c_uint64), ("e_offset", ctypes.c_uint64),
                ("chunk_values", ctypes.c_uint32), ("stream_values", ctypes.c_uint32), ("n_chunks", ctypes.c_uint32),
                ("max_len", ctypes.c_uint32), ("lane_quantum", ctypes.c_uint32), ("n_present", ctypes.c_uint32),
                ("table_stride", ctypes.c_uint32), ("reserved", ctypes.c_uint32)]


class TensorParts(ctypes.Structure):
    """zm_tensor_parts"""
    _fields_ = [("table", ctypes.c_void_p), ("chunk_offsets", ctypes.c_void_p), ("sm", ctypes.c_void_p),
                ("echunks", ctypes.c_void_p)]


class LaunchShape(ctypes.Structure):
    """zm_launch_shape"""
    _fields_ = [("round_symbols", ctypes.c_uint32), ("waves_per_workgroup", ctypes.c_uint32),
                ("streaming_stores", ctypes.c_uint32), ("workgroups", ctypes.c_uint32), ("tensors", ctypes.c_uint32),
                ("lds_bytes", ctypes.c_uint32)]


class CacheConfig(ctypes.Structure):
    """zm_cache_config"""
    _fields_ = [("n_experts", ctypes.c_int32), ("tensors_per_expert", ctypes.c_int32), ("slots", ctypes.c_int32 * 4),
                ("tolerance", ctypes.c_int32), ("max_selected", ctypes.c_int32)]


class SchedTask(ctypes.Structure):
    """zm_sched_task"""
    _fields_ = [("expert", ctypes.c_int32), ("needs_sm", ctypes.c_int32), ("needs_e", ctypes.c_int32),
                ("needs_decode", ctypes.c_int32)]


class SchedCosts(ctypes.Structure):
    """zm_sched_costs"""
    _fields_ = [("sm_read", ctypes.c_double), ("e_read", ctypes.c_double), ("decompress", ctypes.c_double),
                ("recover", ctypes.c_double), ("threads", ctypes.c_int32), ("shards", ctypes.c_int32)]


class SchedEvent(ctypes.Structure):
    """zm_sched_event"""
    _fields_ = [("kind", ctypes.c_int32), ("task", ctypes.c_int32), ("chunk", ctypes.c_int32), ("unit", ctypes.c_int32),
                ("start", ctypes.c_double), ("end", ctypes.c_double)]


class SchedResult(ctypes.Structure):
    """zm_sched_result"""
    _fields_ = [("makespan", ctypes.c_double), ("io_end", ctypes.c_double), ("charge", ctypes.c_double)]


OP_E_READ, OP_SM_READ, OP_DECOMPRESS, OP_RECOVER, OP_EXECUTE = range(5)


class PlanCosts(ctypes.Structure):
    """zm_plan_costs"""
    _fields_ = [("decompress_delay", ctypes.c_double), ("e_read_delay", ctypes.c_double), ("sm_read_delay", ctypes.c_double),
                ("threads", ctypes.c_int32), ("shards_per_tensor", ctypes.c_int32), ("tensors_per_expert", ctypes.c_int32)]


class ZipMoEError(RuntimeError):
    def __init__(self, status: int, where: str):
        super().__init__(f"{where}: {strerror(status)} ({status})")
        self.status = status


_lib: Optional[ctypes.CDLL] = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is not built; run `python -m paper_2601_21198_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        c = ctypes
        u8p, u16p, u64p = c.POINTER(c.c_uint8), c.POINTER(c.c_uint16), c.POINTER(c.c_uint64)
        L.zm_version.argtypes = []
        L.zm_version.restype = c.c_int
        L.zm_strerror.argtypes = [c.c_int]
        L.zm_strerror.restype = c.c_char_p
        L.zm_exponent_histogram.argtypes = [u16p, c.c_size_t, u64p]
        L.zm_build_codebook.argtypes = [u64p, c.c_int, u8p]
        L.zm_encode_bound.argtypes = [c.c_size_t, c.c_uint32, c.c_uint32]
        L.zm_encode_bound.restype = c.c_size_t
        L.zm_encode.argtypes = [u16p, c.c_size_t, c.c_uint32, c.c_uint32, u8p, u8p, c.c_size_t,
                                c.POINTER(c.c_size_t), u64p, c.c_size_t, c.POINTER(c.c_size_t)]
        L.zm_blob_info.argtypes = [c.c_void_p, c.c_size_t, c.POINTER(TensorInfo)]
        L.zm_validate_blob.argtypes = [c.c_void_p, c.c_size_t]
        L.zm_decode_experts.argtypes = [c.POINTER(c.c_void_p), c.POINTER(c.c_void_p), c.POINTER(TensorInfo),
                                        c.c_int, c.c_int, c.POINTER(c.c_int32), c.c_int,
                                        c.POINTER(c.c_void_p), c.c_void_p]
        L.zm_decode_experts_stores.argtypes = [c.POINTER(c.c_void_p), c.POINTER(c.c_void_p), c.POINTER(TensorInfo),
                                               c.c_int, c.c_int, c.POINTER(c.c_int32), c.c_int,
                                               c.POINTER(c.c_void_p), c.c_int, c.c_void_p]
        L.zm_decode_launch_shapes.argtypes = [c.POINTER(TensorInfo), c.c_int, c.c_int, c.POINTER(LaunchShape), c.c_int,
                                              c.POINTER(c.c_int)]
        L.zm_decode_tensors.argtypes = [c.POINTER(TensorParts), c.POINTER(TensorInfo), c.c_int,
                                        c.POINTER(c.c_void_p), c.c_void_p]
        L.zm_decode_host_tensors.argtypes = [c.POINTER(c.c_void_p), c.POINTER(TensorInfo), c.c_int,
                                             c.POINTER(c.c_void_p), c.c_void_p]
        L.zm_decode_exponents_host.argtypes = [c.c_void_p, c.c_size_t, c.c_uint32, c.c_uint32, u8p, c.c_int]
        L.zm_mover_probe.argtypes = [c.c_void_p, c.c_void_p, c.c_size_t, c.c_size_t, c.c_int, c.c_int, c.c_void_p]
        L.zm_recover.argtypes = [c.c_void_p, c.c_void_p, c.c_size_t, c.c_void_p, c.c_void_p]
        L.zm_layer_arena_bytes.argtypes = [c.POINTER(c.c_size_t), c.c_int, c.POINTER(c.c_size_t)]
        L.zm_layer_create.argtypes = [c.POINTER(c.c_void_p), c.POINTER(c.c_size_t), c.c_int, c.c_int, c.c_void_p, c.c_size_t,
                                      c.POINTER(c.c_void_p)]
        L.zm_layer_tensor_info.argtypes = [c.c_void_p, c.c_int, c.c_int, c.POINTER(TensorInfo), c.POINTER(c.c_void_p)]
        L.zm_layer_decode.argtypes = [c.c_void_p, c.POINTER(c.c_int32), c.c_int, c.POINTER(c.c_void_p), c.c_int, c.c_void_p]
        L.zm_layer_destroy.argtypes = [c.c_void_p]
        L.zm_layer_destroy.restype = None
        L.zm_cache_dispatch.argtypes = [u64p, c.c_int, c.POINTER(c.c_int32), c.c_int, c.c_int]
        L.zm_cache_arena_bytes.argtypes = [c.POINTER(CacheConfig), c.POINTER(TensorInfo), c.POINTER(c.c_size_t)]
        L.zm_cache_image_bytes.argtypes = [c.POINTER(CacheConfig), c.POINTER(TensorInfo), c.POINTER(c.c_size_t)]
        L.zm_cache_pack_expert.argtypes = [c.POINTER(CacheConfig), c.POINTER(TensorInfo), c.POINTER(c.c_void_p), c.c_int,
                                           c.c_void_p, c.c_size_t]
        L.zm_cache_create.argtypes = [c.POINTER(CacheConfig), c.POINTER(c.c_void_p), c.POINTER(c.c_void_p),
                                      c.POINTER(TensorInfo), c.c_void_p,
                                      c.c_size_t, c.POINTER(c.c_void_p)]
        L.zm_cache_fetch.argtypes = [c.c_void_p, c.POINTER(c.c_int32), c.c_int, c.POINTER(c.c_void_p),
                                     c.POINTER(c.c_int32), c.c_void_p]
        L.zm_cache_pool_of.argtypes = [c.c_void_p, c.c_int]
        L.zm_cache_destroy.argtypes = [c.c_void_p]
        L.zm_cache_destroy.restype = None
        dp = c.POINTER(c.c_double)
        L.zm_plan_selection_probabilities.argtypes = [dp, c.c_int, c.c_int, c.c_int, c.c_double, dp, c.POINTER(c.c_int)]
        L.zm_plan_hit_distribution.argtypes = [dp, c.c_int, dp]
        L.zm_plan_makespan.argtypes = [c.c_int, c.POINTER(c.c_int32), c.POINTER(PlanCosts), dp]
        L.zm_plan_expected_makespan.argtypes = [dp, c.c_int, c.POINTER(c.c_int32), c.c_int, c.POINTER(PlanCosts), dp]
        L.zm_plan_pools.argtypes = [dp, c.c_int, c.c_int, c.POINTER(PlanCosts), c.c_double, dp, c.c_int, c.c_int,
                                    dp, c.POINTER(c.c_int32), dp]
        for name in EXPORTS:
            if name not in ("zm_strerror", "zm_encode_bound", "zm_cache_destroy", "zm_layer_destroy"):
                getattr(L, name).restype = c.c_int
        _lib = L
    return _lib


def _check(status: int, where: str) -> None:
    if status != OK:
        raise ZipMoEError(status, where)


def _ptr(a: np.ndarray, t):
    return a.ctypes.data_as(ctypes.POINTER(t))


def version() -> int:
    return int(lib().zm_version())


def strerror(status: int) -> str:
    return lib().zm_strerror(status).decode()


def _words(bf16) -> np.ndarray:
    a = np.ascontiguousarray(bf16)
    if a.dtype != np.uint16:
        raise TypeError("bf16 values are passed as their uint16 bit patterns")
    return a.reshape(-1)


def exponent_histogram(bf16) -> np.ndarray:
    w = _words(bf16)
    hist = np.zeros(256, np.uint64)
    _check(lib().zm_exponent_histogram(_ptr(w, ctypes.c_uint16), w.size, _ptr(hist, ctypes.c_uint64)),
           "zm_exponent_histogram")
    return hist


def build_codebook(hist, max_len: int = 8) -> np.ndarray:
    h = np.ascontiguousarray(hist, np.uint64)
    if h.shape != (256,):
        raise ValueError("hist must have 256 entries")
    out = np.zeros(256, np.uint8)
    _check(lib().zm_build_codebook(_ptr(h, ctypes.c_uint64), int(max_len), _ptr(out, ctypes.c_uint8)),
           "zm_build_codebook")
    return out


def encode_bound(n_values: int, chunk_values: int, stream_values: int) -> int:
    return int(lib().zm_encode_bound(n_values, chunk_values, stream_values))


def encode(bf16, chunk_values: int, stream_values: int, code_len) -> Tuple[np.ndarray, np.ndarray]:
    """zm_encode: returns (blob as uint8 array, chunk table as uint64 array shaped [n_chunks+1, table_stride/8]:
    column 0 is the offset|mode word of every chunk, the last row holds the end offset)."""
    w = _words(bf16)
    cl = np.ascontiguousarray(code_len, np.uint8)
    cap = encode_bound(w.size, chunk_values, stream_values)
    if cap == 0:
        raise ZipMoEError(E_ARG, "zm_encode_bound")
    blob = np.empty(cap, np.uint8)
    max_chunks = -(-w.size // chunk_values) + 1
    words_per_entry = -(-(8 + 4 * (chunk_values // stream_values + 1)) // 8)
    offs = np.zeros(max_chunks * words_per_entry, np.uint64)
    size, n_chunks = ctypes.c_size_t(0), ctypes.c_size_t(0)
    _check(lib().zm_encode(_ptr(w, ctypes.c_uint16), w.size, chunk_values, stream_values, _ptr(cl, ctypes.c_uint8),
                           _ptr(blob, ctypes.c_uint8), cap, ctypes.byref(size),
                           _ptr(offs, ctypes.c_uint64), offs.size, ctypes.byref(n_chunks)), "zm_encode")
    return blob[: size.value].copy(), offs[: (n_chunks.value + 1) * words_per_entry].reshape(-1, words_per_entry).copy()


def compress(bf16, chunk_values: int, stream_values: int = 4096, max_len: int = 8) -> Tuple[np.ndarray, np.ndarray]:
    """histogram -> codebook -> encode: the offline initialisation of one tensor."""
    w = _words(bf16)
    return encode(w, chunk_values, stream_values, build_codebook(exponent_histogram(w), max_len))


def blob_info(blob) -> TensorInfo:
    b = np.ascontiguousarray(blob, np.uint8)
    info = TensorInfo()
    _check(lib().zm_blob_info(b.ctypes.data, b.size, ctypes.byref(info)), "zm_blob_info")
    return info


def validate_blob(blob) -> None:
    b = np.ascontiguousarray(blob, np.uint8)
    _check(lib().zm_validate_blob(b.ctypes.data, b.size), "zm_validate_blob")


def decode_experts(blobs, chunk_offsets, infos, n_experts: int, tensors_per_expert: int,
                   expert_ids, n_selected: int, out_bf16, stream: int = 0) -> None:
    """zm_decode_experts with ready-made ctypes arrays (see ``ExpertLayer`` for a convenient owner)."""
    _check(lib().zm_decode_experts(blobs, chunk_offsets, infos, n_experts, tensors_per_expert,
                                   expert_ids, n_selected, out_bf16, ctypes.c_void_p(stream)), "zm_decode_experts")


def decode_exponents_host(blob, chunk_begin: int = 0, chunk_end: Optional[int] = None, n_threads: int = 1,
                          out: Optional[np.ndarray] = None) -> np.ndarray:
    """zm_decode_exponents_host: exponent bytes of chunks [chunk_begin, chunk_end) (default: all)."""
    b = np.ascontiguousarray(blob, np.uint8)
    info = blob_info(b[:384])
    if chunk_end is None:
        chunk_end = int(info.n_chunks)
    if out is None:
        out = np.zeros(int(info.n_values), np.uint8)
    assert out.dtype == np.uint8 and out.flags.c_contiguous and out.size >= int(info.n_values)
    _check(lib().zm_decode_exponents_host(b.ctypes.data, b.size, chunk_begin, chunk_end,
                                          _ptr(out, ctypes.c_uint8), n_threads), "zm_decode_exponents_host")
    return out


def recover(exponents_ptr: int, sign_mantissa_ptr: int, n_values: int, out_ptr: int, stream: int = 0) -> None:
    """zm_recover on device pointers."""
    _check(lib().zm_recover(ctypes.c_void_p(exponents_ptr), ctypes.c_void_p(sign_mantissa_ptr), n_values,
                            ctypes.c_void_p(out_ptr), ctypes.c_void_p(stream)), "zm_recover")


def mover_probe(src_ptr: int, dst_ptr: int, read_bytes: int, write_bytes: int, pieces_per_lane: int = 1,
                streaming_stores: bool = False, stream: int = 0) -> None:
    """zm_mover_probe on device pointers."""
    _check(lib().zm_mover_probe(ctypes.c_void_p(src_ptr), ctypes.c_void_p(dst_ptr), read_bytes, write_bytes,
                                pieces_per_lane, int(streaming_stores), ctypes.c_void_p(stream)), "zm_mover_probe")


def decode_tensors(parts, infos, n_tensors: int, out_bf16, stream: int = 0) -> None:
    """zm_decode_tensors with ready-made ctypes arrays."""
    _check(lib().zm_decode_tensors(parts, infos, n_tensors, out_bf16, ctypes.c_void_p(stream)), "zm_decode_tensors")


def decode_launch_shapes(infos: Sequence[TensorInfo], stores: int = 0) -> List[LaunchShape]:
    """zm_decode_launch_shapes: the launches a decode call for these tensors would make."""
    n = len(infos)
    arr = (TensorInfo * max(1, n))(*infos)
    out = (LaunchShape * 16)()
    count = ctypes.c_int(0)
    _check(lib().zm_decode_launch_shapes(arr, n, stores, out, 16, ctypes.byref(count)), "zm_decode_launch_shapes")
    return list(out[: min(16, count.value)])


def decode_host_tensors(host_blobs, infos, n_tensors: int, out_bf16, stream: int = 0) -> None:
    """zm_decode_host_tensors with ready-made ctypes arrays."""
    _check(lib().zm_decode_host_tensors(host_blobs, infos, n_tensors, out_bf16, ctypes.c_void_p(stream)),
           "zm_decode_host_tensors")


class ExpertLayer:
    """Owns the device copies of one MoE layer's compressed experts and the pointer tables
    ``zm_decode_experts`` takes.  Holds no arithmetic: it uploads blobs with torch, records their
    device addresses and marshals calls."""

    def __init__(self, expert_blobs: Sequence[Sequence[np.ndarray]], device: str = "cuda:0", validate: bool = True):
        import torch
        self.n_experts = len(expert_blobs)
        self.tensors_per_expert = len(expert_blobs[0])
        n = self.n_experts * self.tensors_per_expert
        self.infos = (TensorInfo * n)()
        self.blob_ptrs = (ctypes.c_void_p * n)()
        self.table_ptrs = (ctypes.c_void_p * n)()
        self.device = torch.device(device)
        self.compressed_bytes = 0
        sizes = []
        for e, tensors in enumerate(expert_blobs):
            assert len(tensors) == self.tensors_per_expert
            for m, blob in enumerate(tensors):
                if validate:
                    validate_blob(blob)
                self.infos[e * self.tensors_per_expert + m] = blob_info(blob[:384])
                sizes.append(int(blob.size))
        # one contiguous arena for the whole layer (blob sizes are multiples of 256, so every blob stays aligned)
        self.arena = torch.empty(sum(sizes), dtype=torch.uint8, device=self.device)
        at = 0
        k = 0
        for tensors in expert_blobs:
            for blob in tensors:
                self.arena[at: at + blob.size].copy_(torch.from_numpy(np.ascontiguousarray(blob)))
                base = self.arena.data_ptr() + at
                self.blob_ptrs[k] = base
                self.table_ptrs[k] = base + self.infos[k].table_offset
                at += blob.size
                k += 1
        self.compressed_bytes = at
        self._ptr_blobs = ctypes.cast(self.blob_ptrs, ctypes.POINTER(ctypes.c_void_p))
        self._ptr_tables = ctypes.cast(self.table_ptrs, ctypes.POINTER(ctypes.c_void_p))
        self._ptr_infos = ctypes.cast(self.infos, ctypes.POINTER(TensorInfo))

    def expert_values(self, expert: int) -> List[int]:
        t = self.tensors_per_expert
        return [int(self.infos[expert * t + m].n_values) for m in range(t)]

    def alloc_outputs(self, n_selected: int, expert: int = 0):
        """One uint16 device tensor per selected slot, tensors of an expert back to back (16-byte aligned each)."""
        import torch
        vals = self.expert_values(expert)
        starts, at = [], 0
        for v in vals:
            starts.append(at)
            at += -(-v // 8) * 8
        bufs = [torch.empty(at, dtype=torch.int16, device=self.device) for _ in range(n_selected)]
        return bufs, starts, vals

    def make_call(self, expert_ids, out_buffers, starts, stores: int = STORES_AUTO):
        """Pre-marshals one call: returns a zero-argument function that enqueues it on ``stream``."""
        ids = (ctypes.c_int32 * len(expert_ids))(*[int(e) for e in expert_ids])
        t = self.tensors_per_expert
        outs = (ctypes.c_void_p * (len(expert_ids) * t))()
        for j, buf in enumerate(out_buffers):
            for m in range(t):
                outs[j * t + m] = buf.data_ptr() + 2 * starts[m]
        f = lib().zm_decode_experts_stores
        args = (self._ptr_blobs, self._ptr_tables, self._ptr_infos, self.n_experts, t, ids, len(expert_ids), outs, stores)

        def call(stream: int = 0):
            rc = f(*args, ctypes.c_void_p(stream))
            if rc != OK:
                raise ZipMoEError(rc, "zm_decode_experts_stores")
        call.keepalive = (ids, outs, out_buffers)
        return call

    def decode(self, expert_ids, out_buffers, starts, stream: int = 0, stores: int = STORES_AUTO) -> None:
        self.make_call(expert_ids, out_buffers, starts, stores)(stream)


class Layer:
    """zm_layer: the library's own handle for one layer's resident experts.  The arena is a torch tensor this
    object keeps alive; everything else is argument marshalling."""

    def __init__(self, expert_blobs: Sequence[Sequence[np.ndarray]], device: str = "cuda:0"):
        import torch
        self.n_experts = len(expert_blobs)
        self.tensors_per_expert = len(expert_blobs[0])
        flat = [np.ascontiguousarray(b, np.uint8) for tensors in expert_blobs for b in tensors]
        n = len(flat)
        sizes = (ctypes.c_size_t * n)(*[int(b.size) for b in flat])
        need = ctypes.c_size_t(0)
        _check(lib().zm_layer_arena_bytes(sizes, n, ctypes.byref(need)), "zm_layer_arena_bytes")
        self.arena = torch.empty(need.value, dtype=torch.uint8, device=torch.device(device))
        ptrs = (ctypes.c_void_p * n)(*[b.ctypes.data for b in flat])
        handle = ctypes.c_void_p(None)
        _check(lib().zm_layer_create(ptrs, sizes, self.n_experts, self.tensors_per_expert,
                                     ctypes.c_void_p(self.arena.data_ptr()), need.value, ctypes.byref(handle)), "zm_layer_create")
        self._handle = handle

    def tensor_info(self, expert: int, tensor: int) -> TensorInfo:
        info = TensorInfo()
        _check(lib().zm_layer_tensor_info(self._handle, expert, tensor, ctypes.byref(info), None), "zm_layer_tensor_info")
        return info

    def decode(self, expert_ids, out_ptrs, stream: int = 0, stores: int = STORES_AUTO) -> None:
        """out_ptrs: device addresses, one per selected expert and tensor (expert-major)."""
        ids = (ctypes.c_int32 * len(expert_ids))(*[int(e) for e in expert_ids])
        outs = (ctypes.c_void_p * len(out_ptrs))(*[int(p) for p in out_ptrs])
        _check(lib().zm_layer_decode(self._handle, ids, len(expert_ids), outs, stores, ctypes.c_void_p(stream)), "zm_layer_decode")

    def close(self) -> None:
        if self._handle:
            lib().zm_layer_destroy(self._handle)
            self._handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def cache_dispatch(counts, slots, tolerance: int, expert: int) -> int:
    """zm_cache_dispatch: the pool the rank rule of Sec. 3.4 assigns to ``expert``."""
    cnt = np.ascontiguousarray(counts, np.uint64)
    sl = (ctypes.c_int32 * 4)(*[int(x) for x in slots])
    rc = lib().zm_cache_dispatch(_ptr(cnt, ctypes.c_uint64), cnt.size, sl, tolerance, expert)
    if rc < 0:
        raise ZipMoEError(rc, "zm_cache_dispatch")
    return rc


class ExpertCache:
    """Owner of one layer's zm_cache: pins the host blobs, allocates the device arena with torch and
    marshals zm_cache_fetch.  The policy and all data movement are the library's."""

    def __init__(self, expert_blobs: Sequence[Sequence[np.ndarray]], slots, tolerance: int, max_selected: int,
                 device: str = "cuda:0", packed: bool = True):
        """packed: keep one pinned image per expert (zm_cache_pack_expert) so that a fetch copies an expert's
        missing parts in one or two pieces; else the pinned blobs themselves are the tier below HBM."""
        import torch
        self.n_experts = len(expert_blobs)
        self.tensors_per_expert = len(expert_blobs[0])
        n = self.n_experts * self.tensors_per_expert
        self.infos = (TensorInfo * n)()
        self.host = []                       # pinned host memory: the tier below HBM
        ptrs = (ctypes.c_void_p * n)()
        flat = []
        k = 0
        for tensors in expert_blobs:
            for blob in tensors:
                validate_blob(blob)
                self.infos[k] = blob_info(blob[:384])
                if packed:
                    blob = np.ascontiguousarray(blob)
                    flat.append(blob)
                    ptrs[k] = blob.ctypes.data
                else:
                    pinned = torch.empty(blob.size, dtype=torch.uint8, pin_memory=True)
                    pinned.numpy()[:] = blob
                    self.host.append(pinned)
                    ptrs[k] = pinned.data_ptr()
                k += 1
        self.config = CacheConfig(self.n_experts, self.tensors_per_expert, (ctypes.c_int32 * 4)(*[int(x) for x in slots]),
                                  tolerance, max_selected)
        images = None
        if packed:
            size = ctypes.c_size_t(0)
            _check(lib().zm_cache_image_bytes(ctypes.byref(self.config), self.infos, ctypes.byref(size)), "zm_cache_image_bytes")
            images = (ctypes.c_void_p * self.n_experts)()
            for e in range(self.n_experts):
                pinned = torch.empty(size.value, dtype=torch.uint8, pin_memory=True)
                _check(lib().zm_cache_pack_expert(ctypes.byref(self.config), self.infos, ptrs, e,
                                                  ctypes.c_void_p(pinned.data_ptr()), size.value), "zm_cache_pack_expert")
                self.host.append(pinned)
                images[e] = pinned.data_ptr()
        need = ctypes.c_size_t(0)
        _check(lib().zm_cache_arena_bytes(ctypes.byref(self.config), self.infos, ctypes.byref(need)), "zm_cache_arena_bytes")
        self.arena = torch.empty(need.value, dtype=torch.uint8, device=device)
        handle = ctypes.c_void_p()
        _check(lib().zm_cache_create(ctypes.byref(self.config), ptrs, images, self.infos, self.arena.data_ptr(), need.value,
                                     ctypes.byref(handle)), "zm_cache_create")
        self.handle = handle
        self.max_selected = max_selected

    def fetch(self, expert_ids, stream: int = 0):
        """Returns (device pointers [n_selected][tensors_per_expert], pools the experts were found in)."""
        k = len(expert_ids)
        ids = (ctypes.c_int32 * k)(*[int(e) for e in expert_ids])
        outs = (ctypes.c_void_p * (k * self.tensors_per_expert))()
        found = (ctypes.c_int32 * k)()
        _check(lib().zm_cache_fetch(self.handle, ids, k, outs, found, ctypes.c_void_p(stream)), "zm_cache_fetch")
        t = self.tensors_per_expert
        return [[outs[j * t + m] for m in range(t)] for j in range(k)], list(found)

    def pool_of(self, expert: int) -> int:
        rc = lib().zm_cache_pool_of(self.handle, expert)
        if rc < 0:
            raise ZipMoEError(rc, "zm_cache_pool_of")
        return rc

    def close(self) -> None:
        if self.handle:
            lib().zm_cache_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def _dbl(a) -> np.ndarray:
    return np.ascontiguousarray(a, np.float64)


def plan_selection_probabilities(f, k: int, max_iters: int = 5000, tol: float = 1e-12):
    fa = _dbl(f)
    q = np.zeros(fa.size)
    it = ctypes.c_int(0)
    _check(lib().zm_plan_selection_probabilities(_ptr(fa, ctypes.c_double), fa.size, k, max_iters, tol,
                                                 _ptr(q, ctypes.c_double), ctypes.byref(it)), "zm_plan_selection_probabilities")
    return q, it.value


def plan_hit_distribution(q) -> np.ndarray:
    qa = _dbl(q)
    phi = np.zeros(qa.size + 1)
    _check(lib().zm_plan_hit_distribution(_ptr(qa, ctypes.c_double), qa.size, _ptr(phi, ctypes.c_double)), "zm_plan_hit_distribution")
    return phi


def plan_makespan(k: int, hits, costs: PlanCosts) -> float:
    out = ctypes.c_double(0)
    _check(lib().zm_plan_makespan(k, (ctypes.c_int32 * 4)(*hits), ctypes.byref(costs), ctypes.byref(out)), "zm_plan_makespan")
    return out.value


def plan_expected_makespan(q, slots, k: int, costs: PlanCosts) -> float:
    qa = _dbl(q)
    out = ctypes.c_double(0)
    _check(lib().zm_plan_expected_makespan(_ptr(qa, ctypes.c_double), qa.size, (ctypes.c_int32 * 4)(*slots), k,
                                           ctypes.byref(costs), ctypes.byref(out)), "zm_plan_expected_makespan")
    return out.value


def plan_pools(f, k: int, costs: PlanCosts, memory_bytes: float, bytes_per_expert, grid: int, pool_mask: int = 15):
    fa, ba = _dbl(f), _dbl(bytes_per_expert)
    ratios = np.zeros(4)
    slots = (ctypes.c_int32 * 4)()
    cost = ctypes.c_double(0)
    _check(lib().zm_plan_pools(_ptr(fa, ctypes.c_double), fa.size, k, ctypes.byref(costs), memory_bytes,
                               _ptr(ba, ctypes.c_double), grid, pool_mask, _ptr(ratios, ctypes.c_double), slots,
                               ctypes.byref(cost)), "zm_plan_pools")
    return ratios.tolist(), list(slots), cost.value


def _sched_args(tasks, expert_time):
    arr = (SchedTask * max(1, len(tasks)))(*tasks)
    pa = _dbl(expert_time)
    return arr, len(tasks), _ptr(pa, ctypes.c_double), pa.size, pa


def sched_build(tasks, expert_time, costs: SchedCosts):
    """zm_sched_build: returns the blocks as lists of task indices, highest priority first."""
    arr, n, pp, n_exp, keep = _sched_args(tasks, expert_time)
    order = np.zeros(max(1, n), np.int32)
    ends = np.zeros(max(1, n), np.int32)
    n_blocks = ctypes.c_int(0)
    _check(lib().zm_sched_build(arr, n, pp, n_exp, ctypes.byref(costs), _ptr(order, ctypes.c_int32),
                                _ptr(ends, ctypes.c_int32), ctypes.byref(n_blocks)), "zm_sched_build")
    blocks, at = [], 0
    for b in range(n_blocks.value):
        blocks.append(order[at:ends[b]].tolist())
        at = int(ends[b])
    return blocks


def sched_simulate(tasks, expert_time, costs: SchedCosts, blocks, events: bool = True):
    """zm_sched_simulate: returns (SchedResult, worker ends, list of SchedEvent)."""
    arr, n, pp, n_exp, keep = _sched_args(tasks, expert_time)
    order = np.array([j for b in blocks for j in b] or [0], np.int32)
    ends = np.cumsum([len(b) for b in blocks] or [0]).astype(np.int32)
    res = SchedResult()
    worker_end = np.zeros(max(1, costs.threads))
    n_events = ctypes.c_size_t(0)
    L = lib()
    _check(L.zm_sched_simulate(arr, n, pp, n_exp, ctypes.byref(costs), _ptr(order, ctypes.c_int32),
                               _ptr(ends, ctypes.c_int32), len(blocks), ctypes.byref(res),
                               _ptr(worker_end, ctypes.c_double), None, ctypes.c_size_t(0), ctypes.byref(n_events)),
           "zm_sched_simulate")
    if not events:
        return res, worker_end.tolist(), []
    ev = (SchedEvent * max(1, n_events.value))()
    _check(L.zm_sched_simulate(arr, n, pp, n_exp, ctypes.byref(costs), _ptr(order, ctypes.c_int32),
                               _ptr(ends, ctypes.c_int32), len(blocks), ctypes.byref(res),
                               _ptr(worker_end, ctypes.c_double), ev, ctypes.c_size_t(n_events.value), None),
           "zm_sched_simulate")
    return res, worker_end.tolist(), list(ev[:n_events.value])


def sched_lower_bounds(tasks, expert_time, costs: SchedCosts):
    arr, n, pp, n_exp, keep = _sched_args(tasks, expert_time)
    out = np.zeros(4)
    _check(lib().zm_sched_lower_bounds(arr, n, pp, n_exp, ctypes.byref(costs), _ptr(out, ctypes.c_double)),
           "zm_sched_lower_bounds")
    return out.tolist()
