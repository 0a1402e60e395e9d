"""ctypes binding of libconserve_kv with the C names (see include/conserve_kv.h).

Argument marshalling only: torch tensors are used for device memory and streams, every
step of the path runs in the library's kernels.  There is no fallback: if the built
library is missing, loading raises.
"""
import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libconserve_kv.so")

CS_OK = 0
CS_ERR_INVALID_ARG = -1
CS_ERR_UNSUPPORTED = -2
CS_ERR_WORKSPACE_TOO_SMALL = -3
CS_ERR_STAGING_TOO_SMALL = -4
CS_ERR_HIP = -5
CS_ERR_NO_HOST_PAGES = -6
CS_ERR_STATIC_SCRATCH_TOO_SMALL = -7
PAGE = 16


class cs_kv_pool(ctypes.Structure):
    _fields_ = [
        ("base", ctypes.c_void_p),
        ("num_layers", ctypes.c_int32),
        ("num_pages", ctypes.c_int32),
        ("page_size", ctypes.c_int32),
        ("num_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32),
        ("layer_stride", ctypes.c_int64),
        ("page_stride", ctypes.c_int64),
    ]


class cs_batch(ctypes.Structure):
    _fields_ = [
        ("num_seqs", ctypes.c_int32),
        ("num_tokens", ctypes.c_int32),
        ("block_tables", ctypes.c_void_p),
        ("max_blocks_per_seq", ctypes.c_int32),
        ("ctx_lens", ctypes.c_void_p),
        ("cu_q_lens", ctypes.c_void_p),
        ("h_ctx_lens", ctypes.c_void_p),
        ("h_cu_q_lens", ctypes.c_void_p),
    ]


POLL_FN = ctypes.CFUNCTYPE(ctypes.c_int32, ctypes.c_void_p)


class cs_host_store(ctypes.Structure):
    _fields_ = [("base", ctypes.c_void_p), ("num_layers", ctypes.c_int32), ("num_pages", ctypes.c_int32)]


class cs_safepoint(ctypes.Structure):
    _fields_ = [
        ("flag", ctypes.c_void_p),
        ("poll", POLL_FN),
        ("poll_arg", ctypes.c_void_p),
        ("check_every", ctypes.c_int32),
        ("num_online_seqs", ctypes.c_int32),
        ("sync_at_safepoint", ctypes.c_int32),
    ]


class CsError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        msg = lib().cs_status_string(status).decode()
        hip = lib().cs_last_hip_error().decode()
        super().__init__("%s: %s (%d)%s" % (where, msg, status, (" [" + hip + "]") if hip else ""))


_lib = None


def lib():
    """The loaded C library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                "libconserve_kv.so is not built (%s); run `python -m paper_2410_01228_amd.build`" % LIB_PATH)
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
        PP, BP = ctypes.POINTER(cs_kv_pool), ctypes.POINTER(cs_batch)
        L.cs_page_bytes.restype, L.cs_page_bytes.argtypes = sz, [i32, i32]
        L.cs_pool_page_bytes.restype, L.cs_pool_page_bytes.argtypes = sz, [PP]
        L.cs_kv_append.restype, L.cs_kv_append.argtypes = ctypes.c_int, [PP, i32, BP, vp, vp, vp]
        L.cs_paged_attention_workspace_bytes.restype = sz
        L.cs_paged_attention_workspace_bytes.argtypes = [BP, i32, i32, i32]
        for f in (L.cs_paged_attention_mixed, L.cs_paged_attention_mixed_f16):
            f.restype, f.argtypes = ctypes.c_int, [PP, i32, BP, vp, vp, i32, ctypes.c_float, vp, sz, vp]
        L.cs_paged_attention_mixed_static.restype = ctypes.c_int
        L.cs_paged_attention_mixed_static.argtypes = [PP, i32, BP, vp, vp, i32, ctypes.c_float, vp]
        L.cs_static_scratch_bytes.restype, L.cs_static_scratch_bytes.argtypes = sz, []
        for f in (L.cs_kv_ckpt_gather, L.cs_kv_ckpt_restore, L.cs_kv_ckpt_gather_tokens, L.cs_kv_ckpt_restore_tokens):
            f.restype, f.argtypes = ctypes.c_int, [PP, i32, i32, vp, i32, vp, sz, vp]
        for f in (L.cs_kv_ckpt_save, L.cs_kv_ckpt_load):
            f.restype, f.argtypes = ctypes.c_int, [PP, i32, i32, vp, i32, vp, sz, vp, vp]
        for f in (L.cs_kv_ckpt_save_run, L.cs_kv_ckpt_load_run):
            f.restype, f.argtypes = ctypes.c_int, [PP, i32, i32, vp, i32, vp, sz, ctypes.POINTER(cs_host_store), i32, vp]
        ip = ctypes.POINTER(ctypes.c_int32)
        L.cs_page_map_create.restype, L.cs_page_map_create.argtypes = vp, [i32, i32]
        L.cs_page_map_destroy.restype, L.cs_page_map_destroy.argtypes = None, [vp]
        L.cs_page_map_host_of.restype, L.cs_page_map_host_of.argtypes = i32, [vp, i32]
        L.cs_page_map_gpu_of.restype, L.cs_page_map_gpu_of.argtypes = i32, [vp, i32]
        L.cs_page_map_free_host_pages.restype, L.cs_page_map_free_host_pages.argtypes = i32, [vp]
        L.cs_page_map_checkpoint.restype, L.cs_page_map_checkpoint.argtypes = i32, [vp, ip, i32, ip, ip]
        L.cs_page_map_evict.restype, L.cs_page_map_evict.argtypes = ctypes.c_int, [vp, ip, i32, ip]
        L.cs_page_map_bind.restype, L.cs_page_map_bind.argtypes = ctypes.c_int, [vp, ip, ip, i32]
        L.cs_page_map_drop.restype, L.cs_page_map_drop.argtypes = ctypes.c_int, [vp, ip, i32]
        L.cs_run_layers_f16.restype = ctypes.c_int
        L.cs_run_layers.restype = ctypes.c_int
        L.cs_run_layers_f16.argtypes = L.cs_run_layers.argtypes = [PP, i32, i32, BP, vp, vp, vp, vp, ctypes.c_int64, ctypes.c_int64, i32,
                                    ctypes.c_float, vp, sz, ctypes.POINTER(cs_safepoint),
                                    ctypes.POINTER(ctypes.c_int32), vp]
        L.cs_run_layers_workspace_bytes.restype = sz
        L.cs_run_layers_workspace_bytes.argtypes = [BP, i32, i32, i32, i32]
        L.cs_debug_set_cu_count.restype, L.cs_debug_set_cu_count.argtypes = None, [i32]
        L.cs_debug_copy.restype, L.cs_debug_copy.argtypes = ctypes.c_int, [vp, vp, sz, vp]
        L.cs_set_decode_split_tokens.restype, L.cs_set_decode_split_tokens.argtypes = None, [i32]
        L.cs_set_mixed_fusion.restype, L.cs_set_mixed_fusion.argtypes = None, [i32]
        L.cs_debug_mixed_arrangement.restype, L.cs_debug_mixed_arrangement.argtypes = i32, [BP, i32, i32, i32]
        L.cs_debug_mixed_tile_priority.restype, L.cs_debug_mixed_tile_priority.argtypes = i32, [BP, i32, i32, i32]
        L.cs_debug_set_tail_cut.restype, L.cs_debug_set_tail_cut.argtypes = None, [i32, i32]
        L.cs_debug_play_tiles.restype = ctypes.c_double
        L.cs_debug_play_tiles.argtypes = [ctypes.POINTER(ctypes.c_float), i32, i32, ctypes.c_double]
        L.cs_debug_mixed_tail_cut.restype = i32
        L.cs_debug_mixed_tail_cut.argtypes = [BP, i32, i32, i32, ctypes.POINTER(i32), ctypes.POINTER(i32)]
        L.cs_set_decode_pages_ahead.restype, L.cs_set_decode_pages_ahead.argtypes = None, [i32]
        L.cs_debug_prefill_order.restype = ctypes.c_int32
        L.cs_debug_prefill_order.argtypes = [BP, i32, i32, i32, ctypes.POINTER(ctypes.c_int32), i32]
        L.cs_debug_decode_pages_ahead.restype, L.cs_debug_decode_pages_ahead.argtypes = ctypes.c_int32, [BP, i32, i32]
        L.cs_debug_decode_items.restype = ctypes.c_int32
        L.cs_debug_decode_items.argtypes = [BP, i32, i32, ctypes.POINTER(ctypes.c_uint32), i32, ctypes.POINTER(ctypes.c_int32)]
        L.cs_status_string.restype, L.cs_status_string.argtypes = ctypes.c_char_p, [ctypes.c_int]
        L.cs_last_hip_error.restype, L.cs_last_hip_error.argtypes = ctypes.c_char_p, []
        _lib = L
    return _lib


EXPORTS = [
    "cs_page_bytes", "cs_pool_page_bytes", "cs_kv_append", "cs_paged_attention_workspace_bytes",
    "cs_paged_attention_mixed", "cs_paged_attention_mixed_f16", "cs_paged_attention_mixed_static", "cs_static_scratch_bytes", "cs_kv_ckpt_gather", "cs_kv_ckpt_restore", "cs_kv_ckpt_gather_tokens",
    "cs_kv_ckpt_restore_tokens", "cs_kv_ckpt_save",
    "cs_kv_ckpt_load", "cs_kv_ckpt_save_run", "cs_kv_ckpt_load_run", "cs_page_map_create", "cs_page_map_destroy",
    "cs_page_map_host_of", "cs_page_map_gpu_of", "cs_page_map_free_host_pages", "cs_page_map_checkpoint",
    "cs_page_map_evict", "cs_page_map_bind", "cs_page_map_drop", "cs_run_layers", "cs_run_layers_f16", "cs_run_layers_workspace_bytes", "cs_debug_set_cu_count", "cs_debug_copy", "cs_debug_decode_items", "cs_debug_decode_pages_ahead", "cs_debug_prefill_order",
    "cs_set_decode_split_tokens", "cs_set_decode_pages_ahead", "cs_set_mixed_fusion", "cs_debug_mixed_arrangement", "cs_debug_mixed_tile_priority", "cs_debug_mixed_tail_cut", "cs_debug_set_tail_cut", "cs_debug_play_tiles", "cs_status_string", "cs_last_hip_error",
]


def _stream(stream) -> int:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, torch.cuda.Stream):
        return stream.cuda_stream
    return int(stream)


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


class Pool:
    """A cs_kv_pool over a torch tensor [L, P, 2, Hkv, page_size*D] bf16 (or any tensor of
    that many elements); keeps the tensor alive."""

    def __init__(self, tensor: torch.Tensor, L: int, P: int, Hkv: int, D: int,
                 layer_stride: Optional[int] = None, page_stride: Optional[int] = None, page_size: int = PAGE):
        self.tensor = tensor
        self.page_size = page_size
        self.page_elems = 2 * Hkv * page_size * D
        ps = self.page_elems if page_stride is None else page_stride
        ls = P * ps if layer_stride is None else layer_stride
        self.c = cs_kv_pool(_ptr(tensor), L, P, page_size, Hkv, D, ls, ps)
        self.L, self.P, self.Hkv, self.D = L, P, Hkv, D

    @classmethod
    def empty(cls, L, P, Hkv, D, device="cuda", page_size: int = PAGE):
        t = torch.empty((L, P, 2, Hkv, page_size * D), dtype=torch.bfloat16, device=device)
        return cls(t, L, P, Hkv, D, page_size=page_size)


class Batch:
    """A cs_batch; device copies are made from the given CPU int32 tensors."""

    def __init__(self, block_tables: torch.Tensor, ctx_lens: torch.Tensor, cu_q_lens: torch.Tensor,
                 device="cuda", num_seqs: Optional[int] = None):
        self.h_bt = block_tables.to(torch.int32).contiguous().cpu()
        self.h_ctx = ctx_lens.to(torch.int32).contiguous().cpu()
        self.h_cu = cu_q_lens.to(torch.int32).contiguous().cpu()
        self.d_bt = self.h_bt.to(device)
        self.d_ctx = self.h_ctx.to(device)
        self.d_cu = self.h_cu.to(device)
        S = self.h_ctx.numel() if num_seqs is None else num_seqs
        self.max_blocks = int(self.h_bt.shape[1]) if self.h_bt.dim() == 2 and self.h_bt.numel() else 1
        self.c = cs_batch(S, int(self.h_cu[S]), _ptr(self.d_bt), self.max_blocks, _ptr(self.d_ctx),
                          _ptr(self.d_cu), _ptr(self.h_ctx), _ptr(self.h_cu))

    def truncated(self, num_seqs: int) -> "Batch":
        """The same arrays with only the first num_seqs sequences (what a layer-wise
        preemption does between two layers; paper Sec. 4.3)."""
        b = object.__new__(Batch)
        b.__dict__.update(self.__dict__)
        b.c = cs_batch(num_seqs, int(self.h_cu[num_seqs]), _ptr(self.d_bt), self.max_blocks,
                       _ptr(self.d_ctx), _ptr(self.d_cu), _ptr(self.h_ctx), _ptr(self.h_cu))
        return b

    @property
    def num_tokens(self):
        return self.c.num_tokens

    @property
    def num_seqs(self):
        return self.c.num_seqs


def _check(rc, where):
    if rc != CS_OK:
        raise CsError(rc, where)


def cs_page_bytes(Hkv: int, D: int) -> int:
    return int(lib().cs_page_bytes(Hkv, D))


def cs_pool_page_bytes(pool: "Pool") -> int:
    return int(lib().cs_pool_page_bytes(ctypes.byref(pool.c)))


def cs_kv_append(pool: Pool, layer: int, batch: Batch, k_new: torch.Tensor, v_new: torch.Tensor, stream=None):
    _check(lib().cs_kv_append(ctypes.byref(pool.c), layer, ctypes.byref(batch.c), _ptr(k_new), _ptr(v_new),
                              _stream(stream)), "cs_kv_append")


def cs_paged_attention_workspace_bytes(batch: Batch, Hq: int, Hkv: int, D: int) -> int:
    return int(lib().cs_paged_attention_workspace_bytes(ctypes.byref(batch.c), Hq, Hkv, D))


def cs_paged_attention_mixed(pool: Pool, layer: int, batch: Batch, q: torch.Tensor, out: torch.Tensor,
                             Hq: int, softmax_scale: float, workspace: Optional[torch.Tensor], stream=None):
    wb = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().cs_paged_attention_mixed(ctypes.byref(pool.c), layer, ctypes.byref(batch.c), _ptr(q), _ptr(out),
                                          Hq, softmax_scale, _ptr(workspace), wb, _stream(stream)),
           "cs_paged_attention_mixed")


def cs_paged_attention_mixed_f16(pool: Pool, layer: int, batch: Batch, q: torch.Tensor, out: torch.Tensor,
                                 Hq: int, softmax_scale: float, workspace: Optional[torch.Tensor], stream=None):
    wb = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().cs_paged_attention_mixed_f16(ctypes.byref(pool.c), layer, ctypes.byref(batch.c), _ptr(q),
                                              _ptr(out), Hq, softmax_scale, _ptr(workspace), wb, _stream(stream)),
           "cs_paged_attention_mixed_f16")


def cs_paged_attention_mixed_static(pool: Pool, layer: int, batch: Batch, q: torch.Tensor, out: torch.Tensor,
                                    Hq: int, softmax_scale: float, stream=None):
    """cs_paged_attention_mixed with the library's own static scratch as workspace (allocates nothing)."""
    _check(lib().cs_paged_attention_mixed_static(ctypes.byref(pool.c), layer, ctypes.byref(batch.c), _ptr(q), _ptr(out),
                                                 Hq, softmax_scale, _stream(stream)), "cs_paged_attention_mixed_static")


def cs_static_scratch_bytes() -> int:
    return int(lib().cs_static_scratch_bytes())


def cs_kv_ckpt_gather(pool: Pool, layer_begin: int, layer_end: int, page_ids: torch.Tensor,
                      staging: torch.Tensor, stream=None):
    _check(lib().cs_kv_ckpt_gather(ctypes.byref(pool.c), layer_begin, layer_end, _ptr(page_ids),
                                   page_ids.numel(), _ptr(staging), staging.numel() * staging.element_size(),
                                   _stream(stream)), "cs_kv_ckpt_gather")


def cs_kv_ckpt_restore(pool: Pool, layer_begin: int, layer_end: int, page_ids: torch.Tensor,
                       staging: torch.Tensor, stream=None):
    _check(lib().cs_kv_ckpt_restore(ctypes.byref(pool.c), layer_begin, layer_end, _ptr(page_ids),
                                    page_ids.numel(), _ptr(staging), staging.numel() * staging.element_size(),
                                    _stream(stream)), "cs_kv_ckpt_restore")


def cs_kv_ckpt_gather_tokens(pool: Pool, layer_begin: int, layer_end: int, token_slots: torch.Tensor,
                             staging: torch.Tensor, stream=None):
    _check(lib().cs_kv_ckpt_gather_tokens(ctypes.byref(pool.c), layer_begin, layer_end, _ptr(token_slots),
                                          token_slots.numel(), _ptr(staging),
                                          staging.numel() * staging.element_size(), _stream(stream)),
           "cs_kv_ckpt_gather_tokens")


def cs_kv_ckpt_restore_tokens(pool: Pool, layer_begin: int, layer_end: int, token_slots: torch.Tensor,
                              staging: torch.Tensor, stream=None):
    _check(lib().cs_kv_ckpt_restore_tokens(ctypes.byref(pool.c), layer_begin, layer_end, _ptr(token_slots),
                                           token_slots.numel(), _ptr(staging),
                                           staging.numel() * staging.element_size(), _stream(stream)),
           "cs_kv_ckpt_restore_tokens")


def cs_kv_ckpt_save(pool: Pool, layer_begin: int, layer_end: int, page_ids: torch.Tensor,
                    staging: torch.Tensor, host_buf: torch.Tensor, stream=None):
    assert host_buf.is_pinned(), "host_buf must be pinned host memory"
    _check(lib().cs_kv_ckpt_save(ctypes.byref(pool.c), layer_begin, layer_end, _ptr(page_ids), page_ids.numel(),
                                 _ptr(staging), staging.numel() * staging.element_size(), _ptr(host_buf),
                                 _stream(stream)), "cs_kv_ckpt_save")


def cs_kv_ckpt_load(pool: Pool, layer_begin: int, layer_end: int, page_ids: torch.Tensor,
                    staging: torch.Tensor, host_buf: torch.Tensor, stream=None):
    assert host_buf.is_pinned(), "host_buf must be pinned host memory"
    _check(lib().cs_kv_ckpt_load(ctypes.byref(pool.c), layer_begin, layer_end, _ptr(page_ids), page_ids.numel(),
                                 _ptr(staging), staging.numel() * staging.element_size(), _ptr(host_buf),
                                 _stream(stream)), "cs_kv_ckpt_load")


class HostStore:
    """A cs_host_store over a pinned CPU tensor [num_pages, num_layers, page_elems]."""

    def __init__(self, tensor: torch.Tensor):
        assert tensor.is_pinned() and tensor.is_contiguous() and tensor.dim() == 3
        self.tensor = tensor
        self.c = cs_host_store(_ptr(tensor), int(tensor.shape[1]), int(tensor.shape[0]))


class PageMap:
    """cs_page_map: which host page holds the checkpoint of a GPU page (host bookkeeping)."""

    def __init__(self, num_gpu_pages: int, num_host_pages: int):
        self._h = lib().cs_page_map_create(num_gpu_pages, num_host_pages)
        if not self._h:
            raise CsError(CS_ERR_INVALID_ARG, "cs_page_map_create")

    def close(self):
        if getattr(self, "_h", None) and _lib is not None:
            _lib.cs_page_map_destroy(self._h)
        self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @staticmethod
    def _arr(xs):
        return (ctypes.c_int32 * max(1, len(xs)))(*xs)

    def host_of(self, gpu_page: int) -> int:
        return int(lib().cs_page_map_host_of(self._h, gpu_page))

    def gpu_of(self, host_page: int) -> int:
        return int(lib().cs_page_map_gpu_of(self._h, host_page))

    def free_host_pages(self) -> int:
        return int(lib().cs_page_map_free_host_pages(self._h))

    def checkpoint(self, gpu_pages):
        """-> (pages that need saving, first host page of their run); raises CsError."""
        gpu_pages = list(gpu_pages)
        dirty = self._arr([0] * len(gpu_pages))
        first = ctypes.c_int32(-1)
        n = lib().cs_page_map_checkpoint(self._h, self._arr(gpu_pages), len(gpu_pages), dirty, ctypes.byref(first))
        if n < 0:
            raise CsError(n, "cs_page_map_checkpoint")
        return [int(dirty[i]) for i in range(n)], int(first.value)

    def evict(self, gpu_pages):
        gpu_pages = list(gpu_pages)
        out = self._arr([0] * len(gpu_pages))
        _check(lib().cs_page_map_evict(self._h, self._arr(gpu_pages), len(gpu_pages), out), "cs_page_map_evict")
        return [int(out[i]) for i in range(len(gpu_pages))]

    def bind(self, host_pages, gpu_pages):
        host_pages, gpu_pages = list(host_pages), list(gpu_pages)
        assert len(host_pages) == len(gpu_pages)
        _check(lib().cs_page_map_bind(self._h, self._arr(host_pages), self._arr(gpu_pages), len(host_pages)), "cs_page_map_bind")

    def drop(self, host_pages):
        host_pages = list(host_pages)
        _check(lib().cs_page_map_drop(self._h, self._arr(host_pages), len(host_pages)), "cs_page_map_drop")


def ascending_runs(pages):
    """Split a list of host pages into maximal runs p, p+1, ...: [(start index, length)]."""
    runs, i = [], 0
    while i < len(pages):
        j = i + 1
        while j < len(pages) and pages[j] == pages[j - 1] + 1:
            j += 1
        runs.append((i, j - i))
        i = j
    return runs


def cs_kv_ckpt_save_run(pool: Pool, layer_begin: int, layer_end: int, page_ids: torch.Tensor,
                        staging: torch.Tensor, store: HostStore, first_host_page: int, stream=None):
    _check(lib().cs_kv_ckpt_save_run(ctypes.byref(pool.c), layer_begin, layer_end, _ptr(page_ids), page_ids.numel(),
                                     _ptr(staging), staging.numel() * staging.element_size(), ctypes.byref(store.c),
                                     first_host_page, _stream(stream)), "cs_kv_ckpt_save_run")


def cs_kv_ckpt_load_run(pool: Pool, layer_begin: int, layer_end: int, page_ids: torch.Tensor,
                        staging: torch.Tensor, store: HostStore, first_host_page: int, stream=None):
    _check(lib().cs_kv_ckpt_load_run(ctypes.byref(pool.c), layer_begin, layer_end, _ptr(page_ids), page_ids.numel(),
                                     _ptr(staging), staging.numel() * staging.element_size(), ctypes.byref(store.c),
                                     first_host_page, _stream(stream)), "cs_kv_ckpt_load_run")


def cs_run_layers(pool: Pool, layer_begin: int, layer_end: int, batch: Batch, q: torch.Tensor,
                  k_new: torch.Tensor, v_new: torch.Tensor, out: torch.Tensor, Hq: int, softmax_scale: float,
                  workspace: Optional[torch.Tensor], safepoint: Optional[cs_safepoint] = None, stream=None,
                  f16: bool = False) -> int:
    """q, out: [layers, T, Hq, D]; k_new, v_new: [layers, T, Hkv, D].  Returns the first layer
    that ran online-only, or -1.  f16: the data is fp16 (cs_run_layers_f16)."""
    wb = 0 if workspace is None else workspace.numel() * workspace.element_size()
    first = ctypes.c_int32(-1)
    fn = lib().cs_run_layers_f16 if f16 else lib().cs_run_layers
    _check(fn(ctypes.byref(pool.c), layer_begin, layer_end, ctypes.byref(batch.c), _ptr(q),
                               _ptr(k_new), _ptr(v_new), _ptr(out), q.stride(0), k_new.stride(0), Hq,
                               softmax_scale, _ptr(workspace), wb,
                               ctypes.byref(safepoint) if safepoint is not None else None,
                               ctypes.byref(first), _stream(stream)), "cs_run_layers")
    return first.value


def cs_run_layers_workspace_bytes(batch: Batch, num_online_seqs: int, Hq: int, Hkv: int, D: int) -> int:
    return int(lib().cs_run_layers_workspace_bytes(ctypes.byref(batch.c), num_online_seqs, Hq, Hkv, D))


def run_layers_workspace_for(batch: Batch, num_online_seqs: int, Hq: int, Hkv: int, D: int, device="cuda") -> torch.Tensor:
    n = cs_run_layers_workspace_bytes(batch, num_online_seqs, Hq, Hkv, D)
    return torch.empty(max(n, 16), dtype=torch.uint8, device=device)


def cs_debug_set_cu_count(cus: int):
    lib().cs_debug_set_cu_count(int(cus))


def cs_debug_copy(dst: torch.Tensor, src: torch.Tensor, stream=None):
    nbytes = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() >= nbytes
    _check(lib().cs_debug_copy(_ptr(dst), _ptr(src), nbytes, _stream(stream)), "cs_debug_copy")


def cs_debug_decode_items(batch: "Batch", Hkv: int, D: int, capacity: int = 1024):
    """(items as (seq, piece, pieces) tuples or None when the list does not fit the kernel
    arguments, number of items, target keys per item) -- host only."""
    buf = (ctypes.c_uint32 * capacity)()
    split = ctypes.c_int32(0)
    n = lib().cs_debug_decode_items(ctypes.byref(batch.c), Hkv, D, buf, capacity, ctypes.byref(split))
    if n <= -1000000:
        return None, -1000000 - n, split.value
    if n < 0:
        raise CsError(n, "cs_debug_decode_items")
    return [(w & 0xffff, (w >> 16) & 0xff, w >> 24) for w in buf[:min(n, capacity)]], n, split.value


def cs_set_decode_pages_ahead(pages: int):
    lib().cs_set_decode_pages_ahead(int(pages))


def cs_set_mixed_fusion(mode):
    """1: the host chooses how a mixed batch is launched (default); 0: two kernels in a row; 2: one
    grid, decode work behind the tiles; 3: one grid, a decode workgroup per CU beside the tiles."""
    lib().cs_set_mixed_fusion(int(mode))


def cs_debug_mixed_arrangement(batch: "Batch", Hq: int, Hkv: int, D: int) -> int:
    """0 two kernels, 1 decode behind the tiles, 2 decode beside the tiles -- host only."""
    rc = lib().cs_debug_mixed_arrangement(ctypes.byref(batch.c), Hq, Hkv, D)
    if rc < 0:
        raise CsError(rc, "cs_debug_mixed_arrangement")
    return rc


def cs_debug_mixed_tile_priority(batch: "Batch", Hq: int, Hkv: int, D: int) -> int:
    """The higher of the two issue priorities a fused launch's tile wavefronts alternate between (0: none) -- host only."""
    rc = lib().cs_debug_mixed_tile_priority(ctypes.byref(batch.c), Hq, Hkv, D)
    if rc < 0:
        raise CsError(rc, "cs_debug_mixed_tile_priority")
    return rc


def cs_debug_play_tiles(work_us, cus: int, decode_until_us: float = 0.0) -> float:
    """When the last of the tile workgroups (work_us: microseconds each, beside another tile) ends
    in the host's slot model -- host only."""
    arr = (ctypes.c_float * len(work_us))(*work_us)
    return lib().cs_debug_play_tiles(arr, len(work_us), int(cus), float(decode_until_us))


def cs_debug_set_tail_cut(whole_tiles: int, ranges: int):
    """Force the tail cut of fused mixed launches (whole_tiles < 0: the host decides again)."""
    lib().cs_debug_set_tail_cut(int(whole_tiles), int(ranges))


def cs_debug_mixed_tail_cut(batch: "Batch", Hq: int, Hkv: int, D: int):
    """(tile slots in launch order, launch position from which tiles are cut, ranges of the longest
    cut tile) -- host only."""
    first, ranges = ctypes.c_int32(0), ctypes.c_int32(0)
    n = lib().cs_debug_mixed_tail_cut(ctypes.byref(batch.c), Hq, Hkv, D, ctypes.byref(first), ctypes.byref(ranges))
    if n < 0:
        raise CsError(n, "cs_debug_mixed_tail_cut")
    return n, first.value, ranges.value


def cs_set_decode_split_tokens(tokens: int):
    lib().cs_set_decode_split_tokens(int(tokens))


def workspace_for(batch: Batch, Hq: int, Hkv: int, D: int, device="cuda") -> Optional[torch.Tensor]:
    n = cs_paged_attention_workspace_bytes(batch, Hq, Hkv, D)
    return torch.empty(max(n, 16), dtype=torch.uint8, device=device)
