"""ctypes binding of libpsa.so: the same entry points as include/psa.h, nothing computed here.

torch is used for device memory and streams only.  If the library has not been built the import of
this module still works (so that CPU-only tooling can inspect it) but every call raises: there is
no fallback path of any kind.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libpsa.so")

PSA_F16, PSA_BF16 = 0, 1
PSA_OK = 0
DEVERR_PAGE_RANGE, DEVERR_CTX_RANGE, DEVERR_STALLED = 1, 2, 4


class PsaError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} ({status})")


class _KvDesc(C.Structure):
    _fields_ = [("batch", C.c_int32), ("num_q_heads", C.c_int32), ("num_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("page_size", C.c_int32), ("num_pages", C.c_int32),
                ("max_blocks_per_seq", C.c_int32), ("dtype", C.c_int32),
                ("k_pool", C.c_void_p), ("v_pool", C.c_void_p),
                ("block_table", C.c_void_p), ("ctx_lens", C.c_void_p), ("tier", C.c_void_p)]


class _Tier(C.Structure):
    _fields_ = [("state", C.c_void_p), ("slot_pool", C.c_void_p), ("total_slices", C.c_int64),
                ("num_slots", C.c_int64), ("slice_base", C.c_int64), ("staging", C.c_void_p),
                ("staging_slices", C.c_int64)]


class _Tuning(C.Structure):
    _fields_ = [("chunk_blocks", C.c_int32), ("window_chunks", C.c_int32), ("spin_limit", C.c_int32),
                ("force_bitonic", C.c_int32), ("depth_hint", C.c_void_p),
                ("phase_events", C.c_void_p)]


@dataclass
class Tuning:
    chunk_blocks: int = 0
    window_chunks: int = 0
    spin_limit: int = 0
    force_bitonic: int = 0
    depth_hint: object = None     # int32 device tensor [B][Hkv], or None
    phase_events: object = None   # ctypes array of 6 hipEvent_t (c_void_p), or None

    def c(self) -> _Tuning:
        ev = C.cast(self.phase_events, C.c_void_p) if self.phase_events is not None else None
        hint = self.depth_hint.data_ptr() if self.depth_hint is not None else None
        return _Tuning(self.chunk_blocks, self.window_chunks, self.spin_limit, self.force_bitonic, hint, ev)


_lib = None


def library_path() -> str:
    return _LIB_PATH


def load_library() -> C.CDLL:
    """Loads libpsa.so; raises if it has not been built (python -m paper_2503_00392_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise FileNotFoundError(
                f"{_LIB_PATH} is missing: build it with `python -m paper_2503_00392_amd.build`; "
                "there is no fallback implementation")
        lib = C.CDLL(_LIB_PATH)
        vp, i32, sz, f32 = C.c_void_p, C.c_int32, C.c_size_t, C.c_float
        lib.psa_status_string.restype = C.c_char_p
        lib.psa_status_string.argtypes = [C.c_int]
        lib.psa_decode_workspace_bytes.restype = sz
        lib.psa_decode_workspace_bytes.argtypes = [C.POINTER(_KvDesc), C.POINTER(_Tuning)]
        lib.psa_dense_workspace_bytes.restype = sz
        lib.psa_dense_workspace_bytes.argtypes = [C.POINTER(_KvDesc)]
        lib.psa_build_block_metadata.restype = C.c_int
        lib.psa_build_block_metadata.argtypes = [C.POINTER(_KvDesc), vp, vp, vp, i32, vp]
        lib.psa_build_block_means.restype = C.c_int
        lib.psa_build_block_means.argtypes = [C.POINTER(_KvDesc), vp, vp, vp, i32, vp]
        lib.psa_decode_attention.restype = C.c_int
        lib.psa_decode_attention.argtypes = [C.POINTER(_KvDesc), vp, vp, f32, i32, i32, vp, vp, vp, vp, vp,
                                             vp, vp, vp, C.POINTER(_Tuning), vp, sz, vp]
        lib.psa_decode_attention_static.restype = C.c_int
        lib.psa_decode_attention_static.argtypes = [C.POINTER(_KvDesc), vp, vp, f32, i32, i32, vp, vp, vp, vp, vp,
                                                    vp, vp, C.POINTER(_Tuning), vp]
        lib.psa_append_kv.restype = C.c_int
        lib.psa_append_kv.argtypes = [C.POINTER(_KvDesc), vp, vp, vp, vp, vp]
        lib.psa_topk_attention.restype = C.c_int
        lib.psa_topk_attention.argtypes = [C.POINTER(_KvDesc), vp, vp, i32, i32, vp, vp, vp, vp, vp, vp,
                                           vp, vp, C.POINTER(_Tuning), vp, sz, vp]
        lib.psa_dense_attention.restype = C.c_int
        lib.psa_dense_attention.argtypes = [C.POINTER(_KvDesc), vp, vp, vp, vp, sz, vp]
        lib.psa_tier_state_bytes.restype = sz
        lib.psa_tier_state_bytes.argtypes = [C.c_int64, C.c_int64]
        lib.psa_tier_staging_bytes.restype = sz
        lib.psa_tier_staging_bytes.argtypes = [C.c_int64]
        lib.psa_tier_init.restype = C.c_int
        lib.psa_tier_init.argtypes = [C.POINTER(_Tier), vp]
        lib.psa_tier_update_workspace_bytes.restype = sz
        lib.psa_tier_update_workspace_bytes.argtypes = [C.POINTER(_KvDesc)]
        lib.psa_tier_update.restype = C.c_int
        lib.psa_tier_update.argtypes = [C.POINTER(_KvDesc), vp, vp, C.c_int64, C.c_int64, vp, vp, sz, vp]
        lib.psa_read_device_error.restype = C.c_int
        lib.psa_read_device_error.argtypes = [vp, C.POINTER(C.c_int32), vp]
        _lib = lib
    return _lib


def status_string(status: int) -> str:
    return load_library().psa_status_string(int(status)).decode()


def _ptr(t) -> int | None:
    return None if t is None else t.data_ptr()


def _stream(stream) -> int:
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream


def _dtype_code(dt: torch.dtype) -> int:
    if dt == torch.float16:
        return PSA_F16
    if dt == torch.bfloat16:
        return PSA_BF16
    raise TypeError(f"unsupported element type {dt}")


class Tier:
    """One pool of slots on the GPU shared by the layers of a model whose KV pools live in pinned host
    memory (see psa_tier).  Allocates the state and the slot pool and empties them."""

    def __init__(self, total_slices: int, num_slots: int, device="cuda", stream=None):
        lib = load_library()
        nbytes = int(lib.psa_tier_state_bytes(total_slices, num_slots))
        if nbytes == 0:
            raise ValueError("tier sizes out of range")
        self.total_slices, self.num_slots = int(total_slices), int(num_slots)
        self.state = torch.empty(nbytes, dtype=torch.uint8, device=device)
        self.slot_pool = torch.empty((num_slots, 2, 16, 128), dtype=torch.int16, device=device)
        _check(lib.psa_tier_init(C.byref(self.c(0)), _stream(stream)), "psa_tier_init")

    def c(self, slice_base: int, staging: torch.Tensor | None = None) -> _Tier:
        if staging is None:
            return _Tier(self.state.data_ptr(), self.slot_pool.data_ptr(), self.total_slices, self.num_slots,
                         int(slice_base), None, 0)
        return _Tier(self.state.data_ptr(), self.slot_pool.data_ptr(), self.total_slices, self.num_slots,
                     int(slice_base), staging.data_ptr(), int(staging.staging_slices))

    @staticmethod
    def staging_buffer(slices: int, device="cuda") -> torch.Tensor:
        """A zero-filled staging buffer with room for `slices` slices (see psa_tier.staging): pass it as
        KvCache.staging of the layer whose attention is about to run."""
        nbytes = int(load_library().psa_tier_staging_bytes(int(slices)))
        if nbytes == 0:
            raise ValueError("staging size out of range")
        buf = torch.zeros(nbytes, dtype=torch.uint8, device=device)
        buf.staging_slices = int(slices)
        return buf

    def tables(self):
        """(slot_of [total_slices], owner [num_slots], stamp [num_slots], clock) as host arrays: a look
        into the library's state for tests and statistics."""
        def al(v):
            return (v + 255) // 256 * 256
        raw = self.state.cpu().numpy()
        a = 256
        b = a + al(self.total_slices * 4)
        c = b + al(self.num_slots * 4)
        slot_of = raw[a:a + self.total_slices * 4].view("int32").copy()
        owner = raw[b:b + self.num_slots * 4].view("int32").copy()
        stamp = raw[c:c + self.num_slots * 4].view("uint32").copy()
        return slot_of, owner, stamp, int(raw[:4].view("uint32")[0])


@dataclass
class KvCache:
    """One layer's paged KV cache and its tables (device tensors, see psa_kv_desc).  With `tier` the
    pools are pinned host tensors and `slice_base` is the id of this layer's first slice in the tier."""
    k_pool: torch.Tensor       # [P][Hkv][16][128] fp16 / bf16
    v_pool: torch.Tensor
    block_table: torch.Tensor  # int32 [B][max_blocks]
    ctx_lens: torch.Tensor     # int32 [B]
    num_q_heads: int
    tier: object = None        # Tier or None
    slice_base: int = 0
    staging: object = None     # a Tier.staging_buffer or None (with a tier only)

    def desc(self) -> _KvDesc:
        P, H, T, D = self.k_pool.shape
        assert self.k_pool.is_contiguous() and self.v_pool.is_contiguous()
        assert self.block_table.is_contiguous() and self.block_table.dtype == torch.int32
        assert self.ctx_lens.dtype == torch.int32
        return _KvDesc(self.block_table.shape[0], self.num_q_heads, H, D, T, P,
                       self.block_table.shape[1], _dtype_code(self.k_pool.dtype),
                       _ptr(self.k_pool), _ptr(self.v_pool), _ptr(self.block_table),
                       _ptr(self.ctx_lens), self._tier_ptr())

    def _tier_ptr(self):
        if self.tier is None:
            return None
        assert self.k_pool.is_pinned() and self.v_pool.is_pinned(), "with a tier the pools are pinned host tensors"
        # one struct per cache, kept alive (and in place) for as long as any descriptor may point to it
        key = (id(self.tier), int(self.slice_base), id(self.staging))
        if getattr(self, "_tier_key", None) != key:
            self._tier_c, self._tier_key = self.tier.c(self.slice_base, self.staging), key
        return C.addressof(self._tier_c)


def _check(status: int, where: str) -> None:
    if status != PSA_OK:
        raise PsaError(status, where)


def decode_workspace_bytes(kv: KvCache, tuning: Tuning | None = None) -> int:
    d = kv.desc()
    t = tuning.c() if tuning else None
    return int(load_library().psa_decode_workspace_bytes(C.byref(d), C.byref(t) if t else None))


def dense_workspace_bytes(kv: KvCache) -> int:
    d = kv.desc()
    return int(load_library().psa_dense_workspace_bytes(C.byref(d)))


def build_block_metadata(kv: KvCache, meta: torch.Tensor | None = None, page_fill=None,
                         page_list=None, stream=None) -> torch.Tensor:
    """psa_build_block_metadata; allocates `meta` ([P][Hkv][2][128], the pool's type) if not given."""
    P, H, T, D = kv.k_pool.shape
    if meta is None:
        meta = torch.empty((P, H, 2, D), dtype=kv.k_pool.dtype, device=kv.block_table.device)
    d = kv.desc()
    n_listed = 0 if page_list is None else int(page_list.numel())
    st = load_library().psa_build_block_metadata(C.byref(d), _ptr(meta), _ptr(page_fill), _ptr(page_list),
                                                 n_listed, _stream(stream))
    _check(st, "psa_build_block_metadata")
    return meta


def build_block_means(kv: KvCache, means: torch.Tensor | None = None, page_fill=None, page_list=None,
                      stream=None) -> torch.Tensor:
    """psa_build_block_means; allocates `means` ([P][Hkv][128], the pool's type) if not given."""
    P, H, T, D = kv.k_pool.shape
    if means is None:
        means = torch.empty((P, H, D), dtype=kv.k_pool.dtype, device=kv.block_table.device)
    d = kv.desc()
    n_listed = 0 if page_list is None else int(page_list.numel())
    st = load_library().psa_build_block_means(C.byref(d), _ptr(means), _ptr(page_fill), _ptr(page_list), n_listed,
                                              _stream(stream))
    _check(st, "psa_build_block_means")
    return means


def append_kv(kv: KvCache, k_new: torch.Tensor, v_new: torch.Tensor, meta: torch.Tensor,
              status: torch.Tensor | None = None, stream=None) -> None:
    """psa_append_kv: writes into kv.k_pool, kv.v_pool, kv.ctx_lens and meta in place."""
    assert k_new.is_contiguous() and v_new.is_contiguous() and meta.is_contiguous()
    assert k_new.dtype == kv.k_pool.dtype and v_new.dtype == kv.k_pool.dtype
    d = kv.desc()
    assert tuple(k_new.shape) == (d.batch, d.num_kv_heads, 128) and tuple(v_new.shape) == tuple(k_new.shape)
    st = load_library().psa_append_kv(C.byref(d), _ptr(k_new), _ptr(v_new), _ptr(meta), _ptr(status),
                                      _stream(stream))
    _check(st, "psa_append_kv")


SCORE_UPPER_BOUND, SCORE_CUBOID_CENTER, SCORE_MEAN_KEY = 0, 1, 2      # psa_scorer


@dataclass
class DecodeOutput:
    out: torch.Tensor          # float32 [B][Hq][128]
    n_selected: torch.Tensor   # int32 [B][Hq]
    mass_est: torch.Tensor     # float32 [B][Hq]
    blocks_read: torch.Tensor  # int32 [B][Hkv]
    lse: torch.Tensor          # float32 [B][Hq], natural-log sum of exponentiated logits of the attended tokens
    order: torch.Tensor | None     # int32 [B][Hkv][max_blocks]
    scores: torch.Tensor | None    # float32 [B][Hkv][max_blocks]
    traffic: torch.Tensor | None   # int32 [B][Hkv][2]: K blocks, V blocks loaded


def decode_attention(kv: KvCache, q: torch.Tensor, meta: torch.Tensor, threshold: float,
                     check_granularity: int = 1, *, workspace: torch.Tensor | None = None,
                     outputs: DecodeOutput | None = None, want_order: bool = False,
                     want_scores: bool = False, want_traffic: bool = False,
                     tuning: Tuning | None = None, stream=None, scorer: int = SCORE_UPPER_BOUND) -> DecodeOutput:
    """psa_decode_attention.  Pass `workspace` and `outputs` to make the call allocation-free."""
    d = kv.desc()
    dev = q.device
    B, Hq, H, MB = d.batch, d.num_q_heads, d.num_kv_heads, d.max_blocks_per_seq
    t = tuning.c() if tuning else None
    if workspace is None:
        workspace = torch.empty(max(decode_workspace_bytes(kv, tuning), 256), dtype=torch.uint8, device=dev)
    if outputs is None:
        outputs = DecodeOutput(
            torch.empty((B, Hq, 128), dtype=torch.float32, device=dev),
            torch.empty((B, Hq), dtype=torch.int32, device=dev),
            torch.empty((B, Hq), dtype=torch.float32, device=dev),
            torch.empty((B, H), dtype=torch.int32, device=dev),
            torch.empty((B, Hq), dtype=torch.float32, device=dev),
            torch.empty((B, H, MB), dtype=torch.int32, device=dev) if want_order else None,
            torch.empty((B, H, MB), dtype=torch.float32, device=dev) if want_scores else None,
            torch.empty((B, H, 2), dtype=torch.int32, device=dev) if want_traffic else None)
    o = outputs
    assert q.is_contiguous() and meta.is_contiguous()
    st = load_library().psa_decode_attention(
        C.byref(d), _ptr(q), _ptr(meta), float(threshold), int(check_granularity), int(scorer), _ptr(o.out),
        _ptr(o.n_selected), _ptr(o.mass_est), _ptr(o.blocks_read), _ptr(o.lse), _ptr(o.order),
        _ptr(o.scores), _ptr(o.traffic), C.byref(t) if t else None, _ptr(workspace), workspace.numel(), _stream(stream))
    _check(st, "psa_decode_attention")
    o._workspace = workspace   # keeps the buffer alive until the caller has synchronised
    return o


STATIC_SCRATCH_BYTES = 64 << 20


def decode_attention_static(kv: KvCache, q: torch.Tensor, meta: torch.Tensor, threshold: float,
                            check_granularity: int, outputs: DecodeOutput, *, device_error: torch.Tensor | None = None,
                            tuning: Tuning | None = None, stream=None, scorer: int = SCORE_UPPER_BOUND) -> DecodeOutput:
    """psa_decode_attention_static: the caller brings every output tensor (`outputs.scores` and
    `outputs.traffic` are not written); nothing is allocated here or in the library."""
    d = kv.desc()
    t = tuning.c() if tuning else None
    o = outputs
    st = load_library().psa_decode_attention_static(
        C.byref(d), _ptr(q), _ptr(meta), float(threshold), int(check_granularity), int(scorer), _ptr(o.out),
        _ptr(o.n_selected), _ptr(o.mass_est), _ptr(o.blocks_read), _ptr(o.lse), _ptr(o.order), _ptr(device_error),
        C.byref(t) if t else None, _stream(stream))
    _check(st, "psa_decode_attention_static")
    return o


def topk_attention(kv: KvCache, q: torch.Tensor, meta: torch.Tensor, k_blocks: int, *,
                   workspace: torch.Tensor | None = None, outputs: DecodeOutput | None = None,
                   want_order: bool = False, want_scores: bool = False, want_traffic: bool = False,
                   tuning: Tuning | None = None, stream=None, scorer: int = SCORE_UPPER_BOUND) -> DecodeOutput:
    """psa_topk_attention: the fixed-budget control.  Same buffers as decode_attention."""
    d = kv.desc()
    dev = q.device
    B, Hq, H, MB = d.batch, d.num_q_heads, d.num_kv_heads, d.max_blocks_per_seq
    t = tuning.c() if tuning else None
    if workspace is None:
        workspace = torch.empty(max(decode_workspace_bytes(kv, tuning), 256), dtype=torch.uint8, device=dev)
    if outputs is None:
        outputs = DecodeOutput(
            torch.empty((B, Hq, 128), dtype=torch.float32, device=dev),
            torch.empty((B, Hq), dtype=torch.int32, device=dev),
            torch.empty((B, Hq), dtype=torch.float32, device=dev),
            torch.empty((B, H), dtype=torch.int32, device=dev),
            torch.empty((B, Hq), dtype=torch.float32, device=dev),
            torch.empty((B, H, MB), dtype=torch.int32, device=dev) if want_order else None,
            torch.empty((B, H, MB), dtype=torch.float32, device=dev) if want_scores else None,
            torch.empty((B, H, 2), dtype=torch.int32, device=dev) if want_traffic else None)
    o = outputs
    assert q.is_contiguous() and meta.is_contiguous()
    st = load_library().psa_topk_attention(
        C.byref(d), _ptr(q), _ptr(meta), int(k_blocks), int(scorer), _ptr(o.out), _ptr(o.n_selected), _ptr(o.mass_est),
        _ptr(o.blocks_read), _ptr(o.lse), _ptr(o.order), _ptr(o.scores), _ptr(o.traffic), C.byref(t) if t else None,
        _ptr(workspace), workspace.numel(), _stream(stream))
    _check(st, "psa_topk_attention")
    o._workspace = workspace
    return o


def dense_attention(kv: KvCache, q: torch.Tensor, *, workspace: torch.Tensor | None = None,
                    out: torch.Tensor | None = None, lse: torch.Tensor | None = None, stream=None):
    """psa_dense_attention; returns (out float32 [B][Hq][128], lse float32 [B][Hq])."""
    d = kv.desc()
    dev = q.device
    if workspace is None:
        workspace = torch.empty(max(dense_workspace_bytes(kv), 256), dtype=torch.uint8, device=dev)
    if out is None:
        out = torch.empty((d.batch, d.num_q_heads, 128), dtype=torch.float32, device=dev)
    if lse is None:
        lse = torch.empty((d.batch, d.num_q_heads), dtype=torch.float32, device=dev)
    st = load_library().psa_dense_attention(C.byref(d), _ptr(q), _ptr(out), _ptr(lse), _ptr(workspace),
                                            workspace.numel(), _stream(stream))
    _check(st, "psa_dense_attention")
    out._workspace = workspace
    return out, lse


def tier_state_bytes(total_slices: int, num_slots: int) -> int:
    return int(load_library().psa_tier_state_bytes(total_slices, num_slots))


def tier_staging_bytes(staging_slices: int) -> int:
    return int(load_library().psa_tier_staging_bytes(int(staging_slices)))


def tier_init(tier: Tier, stream=None) -> None:
    _check(load_library().psa_tier_init(C.byref(tier.c(0)), _stream(stream)), "psa_tier_init")


def tier_update_workspace_bytes(kv: KvCache) -> int:
    d = kv.desc()
    return int(load_library().psa_tier_update_workspace_bytes(C.byref(d)))


def tier_update(kv: KvCache, order: torch.Tensor, blocks_read: torch.Tensor, busy_first: int = 0, busy_count: int = 0,
                stats: torch.Tensor | None = None, workspace: torch.Tensor | None = None, stream=None) -> torch.Tensor:
    """Brings the slot pool up to date with the slices the decode call that wrote `order` and
    `blocks_read` used.  Returns `stats` (device int32[5]: hits, misses, placed, evicted, placed from the
    staging buffer)."""
    d = kv.desc()
    dev = order.device
    if workspace is None:
        workspace = torch.empty(tier_update_workspace_bytes(kv), dtype=torch.uint8, device=dev)
    if stats is None:
        stats = torch.zeros(5, dtype=torch.int32, device=dev)
    assert order.dtype == torch.int32 and order.is_contiguous()
    assert blocks_read.dtype == torch.int32 and blocks_read.is_contiguous()
    st = load_library().psa_tier_update(C.byref(d), _ptr(order), _ptr(blocks_read), int(busy_first), int(busy_count),
                                        _ptr(stats), _ptr(workspace), workspace.numel(), _stream(stream))
    _check(st, "psa_tier_update")
    stats._workspace = workspace
    return stats


def read_device_error(workspace: torch.Tensor, stream=None) -> int:
    flags = C.c_int32(0)
    st = load_library().psa_read_device_error(_ptr(workspace), C.byref(flags), _stream(stream))
    _check(st, "psa_read_device_error")
    return int(flags.value)
